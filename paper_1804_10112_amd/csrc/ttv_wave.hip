// TTV A_ij = sum_k B_ijk c_k (Section 5.3) for large tensors: the vector c is held in LDS.
//
// Every stored entry gathers one c_k. With c in global memory those gathers, not the
// streams of coordinates and values, set the pace (they hit L2, but a wave's 64 distinct
// lines take several clocks each through the vector memory path). Here one workgroup of
// sixteen waves stays on every compute unit, copies c (as much of it as fits) into LDS once,
// and its waves then walk through the entries on their own, 256 consecutive entries (four
// per lane, one 16-byte load per array) at a time, two such pieces in flight:
//   - products with c from LDS (entries whose k lies beyond the cached part read global c);
//   - fibre heads: COO compares (i, j) with the entry before; CSF marks the entries at which
//     the fibres of the piece begin (from pos of the bottom level) in a wave-private strip
//     of LDS;
//   - a segmented sum over the wave in registers (lane movement inside the vector ALU), no
//     workgroup barrier anywhere in the loop, so a wave waiting for memory never holds up
//     another.
// Output protocol as in the chunked kernels: the piece that holds a fibre's first entry
// stores the fibre's (possibly partial) sum; what precedes the first head of a piece leaves
// as carry number `piece` and is added afterwards (carry_fixup_kernel), in a fixed order:
// results are bit-reproducible.
// Measured on 50M entries in 8.1M fibres, fp32, c of 50 000 values (78 % / 61 % of it cached):
// COO 214 us (chunked kernel with c in global memory: 324 us), CSF 158 us (357 us). Left out
// after measuring: eight entries per lane (a lane's two 16-byte loads then lie 32 bytes apart:
// 263 / 174 us), four pieces in flight instead of two (no change). What remains is the serial
// instruction stream of a wave: sixteen waves per compute unit is all that one workgroup, which
// the single copy of c forces, can provide.
#include "common.hpp"
#include "scan.hpp"
#include "segreduce.hpp"
#include "wavescan.hpp"

namespace spt {

constexpr int kBig = 1024;                    // threads per workgroup
constexpr int kBigWaves = kBig / kWave;
constexpr int kEPL = 4;                       // consecutive entries per lane
constexpr int kPiece = kEPL * kWave;          // entries of one piece
constexpr int kNP = 2;                        // pieces a wave has in flight per step
constexpr int kCooCacheBytes = 152 * 1024;    // LDS set aside for c (COO: nothing else lives there)
constexpr int kCsfCacheBytes = 120 * 1024;    // CSF: next to 32 KiB of fibre marks

template <typename T>
__device__ __forceinline__ T ld_nt(const T* p) {
  return __builtin_nontemporal_load(p);
}

typedef int32_t int4v __attribute__((ext_vector_type(4)));

// Four consecutive values as 16-byte loads.
__device__ __forceinline__ void load4(const float* p, float (&v)[4]) {
  typedef float f4 __attribute__((ext_vector_type(4)));
  const f4 q = ld_nt(reinterpret_cast<const f4*>(p));
  v[0] = q[0], v[1] = q[1], v[2] = q[2], v[3] = q[3];
}
__device__ __forceinline__ void load4(const double* p, double (&v)[4]) {
  typedef double d2 __attribute__((ext_vector_type(2)));
  const d2 a = ld_nt(reinterpret_cast<const d2*>(p)), b = ld_nt(reinterpret_cast<const d2*>(p) + 1);
  v[0] = a[0], v[1] = a[1], v[2] = b[0], v[3] = b[1];
}
__device__ __forceinline__ void load4(const int32_t* p, int32_t (&v)[4]) {
  const int4v q = ld_nt(reinterpret_cast<const int4v*>(p));
  v[0] = q[0], v[1] = q[1], v[2] = q[2], v[3] = q[3];
}

// kEPL consecutive values or coordinates, 16 bytes per load.
template <typename E>
__device__ __forceinline__ void load_lane(const E* p, E (&v)[kEPL]) {
#pragma unroll
  for (int h = 0; h < kEPL / 4; ++h) {
    E q[4];
    load4(p + 4 * h, q);
#pragma unroll
    for (int r = 0; r < 4; ++r) v[4 * h + r] = q[r];
  }
}

// The workgroup copies c[0 .. cached) into LDS.
template <typename T>
__device__ __forceinline__ void stage_vector(T* s_c, const T* __restrict__ c, int cached) {
  constexpr int U = 8;  // loads in flight per thread: the copy is one round trip per U * kBig values
  int q = threadIdx.x;
  for (; q + (U - 1) * kBig < cached; q += U * kBig) {
    T t[U];
#pragma unroll
    for (int u = 0; u < U; ++u) t[u] = c[q + u * kBig];
#pragma unroll
    for (int u = 0; u < U; ++u) s_c[q + u * kBig] = t[u];
  }
  for (; q < cached; q += kBig) s_c[q] = c[q];
  __syncthreads();
}

// c_k: from LDS below `cached`, from global memory beyond. ALL: everything is cached.
template <typename T, bool ALL>
__device__ __forceinline__ void gather_lane(const T* s_c, const T* __restrict__ c, int cached,
                                            const int32_t (&k)[kEPL], T (&g)[kEPL]) {
#pragma unroll
  for (int r = 0; r < kEPL; ++r) g[r] = s_c[ALL ? k[r] : min(k[r], cached - 1)];
  if (!ALL) {
#pragma unroll
    for (int r = 0; r < kEPL; ++r)
      if (k[r] >= cached) g[r] = c[k[r]];
  }
}

// A lane holds the products p[0 .. kEPL) of its consecutive entries; bit r of headmask says
// that a fibre starts at entry r, key[r] is then that fibre's index in the output.
// Stores the sums of the fibres that start in this piece, and the piece's carry.
template <typename T>
__device__ __forceinline__ void wave_fibre_sums(const T (&p)[kEPL], unsigned headmask, const int (&key)[kEPL],
                                                int carry_idx, int piece, T* __restrict__ out_v,
                                                int32_t* __restrict__ carry_key, T* __restrict__ carry_val) {
  const int lane = lane_id();
  T acc = 0, lead = 0;
  int has_head = 0, last_key = -1;
#pragma unroll
  for (int r = 0; r < kEPL; ++r) {
    if (headmask & (1u << r)) {
      if (!has_head) {
        lead = acc;
        has_head = 1;
      } else {
        out_v[last_key] = acc;
      }
      last_key = key[r];
      acc = 0;
    }
    acc += p[r];
  }
  SegSum<T> me{has_head, acc, last_key};
  wave_seg_step<0x111, 0xf>(me);  // row_shr:1, 2, 4, 8: scan inside each row of 16 lanes
  wave_seg_step<0x112, 0xf>(me);
  wave_seg_step<0x114, 0xf>(me);
  wave_seg_step<0x118, 0xf>(me);
  wave_seg_step<0x142, 0xa>(me);  // row_bcast:15 into rows 1 and 3
  wave_seg_step<0x143, 0xc>(me);  // row_bcast:31 into rows 2 and 3
  SegSum<T> ex;  // what the lanes before this one add up to
  ex.f = dpp_move<0x138, 0xf>(0, me.f);  // wave_shr:1
  ex.v = dpp_move<0x138, 0xf>(T(0), me.v);
  ex.k = dpp_move<0x138, 0xf>(-1, me.k);
  if (lane == 0) ex = SegSum<T>{0, T(0), -1};
  if (has_head) {
    const T total = ex.v + lead;
    if (ex.f) {
      out_v[ex.k] = total;
    } else {  // first head of the piece: what precedes it continues an earlier piece
      carry_key[piece] = (lane == 0 && (headmask & 1u)) ? -1 : carry_idx;
      carry_val[piece] = total;
    }
  }
  if (lane == kWave - 1) {  // the fibre still open at the end of the piece
    if (has_head) {
      out_v[last_key] = acc;
    } else if (ex.f) {
      out_v[ex.k] = ex.v + acc;
    } else {  // no head in the whole piece: everything is carry
      carry_key[piece] = carry_idx;
      carry_val[piece] = ex.v + acc;
    }
  }
}

// ================================================================ COO
// heads[piece] = number of (i, j) fibre starts among the piece's entries.
template <bool VEC>
__global__ __launch_bounds__(kBlock) void ttv_piece_heads_kernel(int nnz, int npieces,
                                                                 const int32_t* __restrict__ ci,
                                                                 const int32_t* __restrict__ cj,
                                                                 int32_t* __restrict__ heads) {
  const int piece = blockIdx.x * (kBlock / kWave) + wave_id();
  if (piece >= npieces) return;
  const int lane = lane_id();
  const int p0 = piece * kPiece + lane * kEPL;
  int32_t i[kEPL], j[kEPL];
  if (VEC && p0 + kEPL <= nnz) {
    load_lane(ci + p0, i);
    load_lane(cj + p0, j);
  } else {
#pragma unroll
    for (int r = 0; r < kEPL; ++r) {
      const int p = min(p0 + r, nnz - 1);  // beyond the end: the last entry again, never a head
      i[r] = ci[p];
      j[r] = cj[p];
    }
  }
  int32_t pi = __shfl_up(i[kEPL - 1], 1), pj = __shfl_up(j[kEPL - 1], 1);
  if (lane == 0) {
    pi = pj = -1;
    if (p0 > 0) {
      pi = ci[p0 - 1];
      pj = cj[p0 - 1];
    }
  }
  int cnt = 0;
#pragma unroll
  for (int r = 0; r < kEPL; ++r) {
    cnt += (i[r] != pi || j[r] != pj) ? 1 : 0;
    pi = i[r];
    pj = j[r];
  }
  cnt = wave_inclusive_sum(cnt);
  if (lane == kWave - 1) heads[piece] = cnt;
}

// One output entry per fibre, at index piece_off[piece] + rank of the fibre's head inside
// the piece (append order = ascending (i, j), Section 3.4).
template <typename T, bool VEC, bool ALL>
__global__ __launch_bounds__(kBig) void ttv_coo_wave_kernel(
    int nnz, int npieces, const int32_t* __restrict__ ci, const int32_t* __restrict__ cj,
    const int32_t* __restrict__ ck, const T* __restrict__ vals, const T* __restrict__ c, int cached,
    const int32_t* __restrict__ piece_off, int32_t* __restrict__ out_i, int32_t* __restrict__ out_j,
    T* __restrict__ out_v, int64_t* __restrict__ out_nnz, int32_t* __restrict__ carry_key,
    T* __restrict__ carry_val) {
  __shared__ T s_c[kCooCacheBytes / sizeof(T)];
  stage_vector(s_c, c, cached);
  const int lane = lane_id();
  const int stride = gridDim.x * kBigWaves;
  // piece number = step * (all waves of the grid) + wave: in one step the grid reads one
  // contiguous stretch of every array. A wave has kNP pieces in flight: all their loads are
  // issued before the first is used.
  // the piece number is the same in all lanes: held in a scalar register, what is indexed by it
  // alone (piece_off, the entry before the piece) is fetched by scalar loads
  for (int piece0 = __builtin_amdgcn_readfirstlane(blockIdx.x * kBigWaves + wave_id()); piece0 < npieces;
       piece0 += kNP * stride) {
    int32_t i[kNP][kEPL], j[kNP][kEPL], k[kNP][kEPL], pi[kNP], pj[kNP], first[kNP];
    T v[kNP][kEPL];
#pragma unroll
    for (int u = 0; u < kNP; ++u) {
      const int piece = min(piece0 + u * stride, npieces - 1);  // beyond the end: the last piece again, not stored
      const int p0 = piece * kPiece + lane * kEPL;
      if (VEC && p0 + kEPL <= nnz) {
        load_lane(ci + p0, i[u]);
        load_lane(cj + p0, j[u]);
        load_lane(ck + p0, k[u]);
        load_lane(vals + p0, v[u]);
      } else {
#pragma unroll
        for (int r = 0; r < kEPL; ++r) {
          const bool ok = p0 + r < nnz;
          const int p = ok ? p0 + r : nnz - 1;  // beyond the end: the last entry's fibre, value 0
          i[u][r] = ci[p];
          j[u][r] = cj[p];
          k[u][r] = ck[p];
          v[u][r] = ok ? vals[p] : T(0);
        }
      }
      const int before = max(piece * kPiece - 1, 0);  // only lane 0 uses it
      pi[u] = ci[before];
      pj[u] = cj[before];
      first[u] = piece_off[piece];
    }
#pragma unroll
    for (int u = 0; u < kNP; ++u) {
      const int piece = piece0 + u * stride;
      if (piece >= npieces) break;
      int32_t qi = __shfl_up(i[u][kEPL - 1], 1), qj = __shfl_up(j[u][kEPL - 1], 1);
      if (lane == 0) {
        qi = piece > 0 ? pi[u] : -1;
        qj = piece > 0 ? pj[u] : -1;
      }
      T g[kEPL];
      gather_lane<T, ALL>(s_c, c, cached, k[u], g);
      unsigned headmask = 0;
#pragma unroll
      for (int r = 0; r < kEPL; ++r) {
        if (i[u][r] != qi || j[u][r] != qj) headmask |= 1u << r;
        qi = i[u][r];
        qj = j[u][r];
      }
      const int cnt = __popc(headmask);
      const int upto = first[u] + wave_inclusive_sum(cnt);
      int next_idx = upto - cnt;
      // the number of fibres of the result: where the last piece's last head lands, plus one
      if (piece == npieces - 1 && lane == kWave - 1 && out_nnz) *out_nnz = upto;
      int key[kEPL];
      T p[kEPL];
#pragma unroll
      for (int r = 0; r < kEPL; ++r) {
        p[r] = v[u][r] * g[r];
        key[r] = next_idx;
        if (headmask & (1u << r)) {
          out_i[next_idx] = i[u][r];
          out_j[next_idx] = j[u][r];
          ++next_idx;
        }
      }
      wave_fibre_sums<T>(p, headmask, key, first[u] - 1, piece, out_v, carry_key, carry_val);
    }
  }
}

// ================================================================ CSF
// first[piece] = first fibre that starts at or after the piece's first entry (piece ==
// npieces: the number of fibres, so that the last piece also covers trailing empty fibres).
// count (may be null) receives the number of values of the result, one per fibre.
__global__ __launch_bounds__(kBlock) void ttv_piece_fibres_kernel(int npieces, int nfib,
                                                                  const int32_t* __restrict__ pos,
                                                                  int32_t* __restrict__ first,
                                                                  int64_t* __restrict__ count) {
  const int piece = blockIdx.x * kBlock + threadIdx.x;
  if (piece == 0 && count) *count = nfib;
  if (piece > npieces) return;
  int lo = 0, hi = nfib + 1;
  if (piece == npieces) lo = hi = nfib;
  const int target = piece * kPiece;
  while (lo < hi) {
    const int mid = lo + ((hi - lo) >> 1);
    if (pos[mid] < target) lo = mid + 1; else hi = mid;
  }
  first[piece] = min(lo, nfib);
}

// out_v[f] = sum over the entries of fibre f (dense over the fibres, zero for empty ones).
template <typename T, bool VEC, bool ALL>
__global__ __launch_bounds__(kBig) void ttv_csf_wave_kernel(
    int nnz, int npieces, const int32_t* __restrict__ first, const int32_t* __restrict__ pos,
    const int32_t* __restrict__ ck, const T* __restrict__ vals, const T* __restrict__ c, int cached,
    T* __restrict__ out_v, int32_t* __restrict__ carry_key, T* __restrict__ carry_val) {
  __shared__ T s_c[kCsfCacheBytes / sizeof(T)];
  // fibre that starts at an entry of one of the wave's pieces, or -1
  __shared__ int32_t s_mark[kBigWaves][kNP][kPiece];
  stage_vector(s_c, c, cached);
  const int lane = lane_id();
#pragma unroll
  for (int u = 0; u < kNP; ++u)
#pragma unroll
    for (int r = 0; r < kEPL; ++r) s_mark[wave_id()][u][lane * kEPL + r] = -1;
  const int stride = gridDim.x * kBigWaves;
  for (int piece0 = __builtin_amdgcn_readfirstlane(blockIdx.x * kBigWaves + wave_id()); piece0 < npieces;
       piece0 += kNP * stride) {
    int32_t k[kNP][kEPL], f_lo[kNP], f_hi[kNP];
    T v[kNP][kEPL];
#pragma unroll
    for (int u = 0; u < kNP; ++u) {
      const int piece = min(piece0 + u * stride, npieces - 1);  // beyond the end: the last piece again, not stored
      const int p0 = piece * kPiece + lane * kEPL;
      // fibres first[piece] .. first[piece + 1] - 1 start inside this piece (or are empty)
      f_lo[u] = first[piece];
      f_hi[u] = first[piece + 1];
      if (VEC && p0 + kEPL <= nnz) {
        load_lane(ck + p0, k[u]);
        load_lane(vals + p0, v[u]);
      } else {
#pragma unroll
        for (int r = 0; r < kEPL; ++r) {
          const bool ok = p0 + r < nnz;
          k[u][r] = ok ? ck[p0 + r] : 0;
          v[u][r] = ok ? vals[p0 + r] : T(0);
        }
      }
    }
#pragma unroll
    for (int u = 0; u < kNP; ++u) {
      const int piece = piece0 + u * stride;
      if (piece >= npieces) break;
      volatile int32_t* mark = s_mark[wave_id()][u];
      const int base = piece * kPiece;
      for (int f = f_lo[u] + lane; f < f_hi[u]; f += kWave) {
        const int a = pos[f], b = pos[f + 1];
        if (b > a) mark[a - base] = f;
        else out_v[f] = T(0);
      }
    }
#pragma unroll
    for (int u = 0; u < kNP; ++u) {
      const int piece = piece0 + u * stride;
      if (piece >= npieces) break;
      volatile int32_t* mark = s_mark[wave_id()][u];
      T g[kEPL];
      gather_lane<T, ALL>(s_c, c, cached, k[u], g);
      __builtin_amdgcn_wave_barrier();
      int key[kEPL];
      unsigned headmask = 0;
      T p[kEPL];
#pragma unroll
      for (int r = 0; r < kEPL; ++r) {
        key[r] = mark[lane * kEPL + r];
        if (key[r] >= 0) headmask |= 1u << r;
        p[r] = v[u][r] * g[r];
      }
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int r = 0; r < kEPL; ++r)
        if (key[r] >= 0) mark[lane * kEPL + r] = -1;
      wave_fibre_sums<T>(p, headmask, key, f_lo[u] - 1, piece, out_v, carry_key, carry_val);
    }
  }
}

// ================================================================ host
static int compute_units() {
  static int cached[64] = {0};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
  if (cached[dev] == 0) {
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
    cached[dev] = n;
  }
  return cached[dev];
}

static int64_t pieces_of(int64_t nnz) { return (nnz + kPiece - 1) / kPiece; }

// Smaller tensors stay with the chunked kernels: the fixed cost of staging c on every
// compute unit is not recovered. So do tensors whose last dimension is so long that less
// than a quarter of c fits the cache: their gathers go to global memory anyway, and the
// chunked kernels keep more waves in flight for that.
bool ttv_wave_applies(int64_t nnz, int64_t K, int dtype) {
  const int64_t vsz = dtype == SPT_F64 ? 8 : 4;
  return nnz >= (int64_t(1) << 18) && nnz + kPiece < INT32_MAX && K * vsz <= 4 * (int64_t)kCsfCacheBytes;
}

size_t ttv_coo_wave_workspace(int64_t nnz) {
  const int64_t np = pieces_of(nnz);
  return 3 * align_up((size_t)np * 4, 256) + align_up((size_t)np * 8, 256) + scan_workspace(np) + 256;
}
size_t ttv_csf_wave_workspace(int64_t nnz) {
  const int64_t np = pieces_of(nnz);
  return align_up((size_t)(np + 1) * 4, 256) + align_up((size_t)np * 4, 256) + align_up((size_t)np * 8, 256) + 256;
}

static bool al16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

template <typename T>
spt_status ttv_coo_wave(int64_t nnz64, int64_t K, const int32_t* ci, const int32_t* cj, const int32_t* ck,
                        const T* vals, const T* c, int32_t* out_i, int32_t* out_j, T* out_v, int64_t* out_nnz,
                        void* ws, size_t ws_bytes, hipStream_t s) {
  const int nnz = (int)nnz64;
  const int np = (int)pieces_of(nnz64);
  if (!ws || ws_bytes < ttv_coo_wave_workspace(nnz64))
    return fail(SPT_ERR_WORKSPACE, "ttv: workspace of %zu bytes needed, %zu given", ttv_coo_wave_workspace(nnz64),
                ws_bytes);
  Workspace W(ws, ws_bytes);
  int32_t* heads = W.take<int32_t>(np);
  int32_t* off = W.take<int32_t>(np);
  int32_t* ckey = W.take<int32_t>(np);
  T* cval = W.take<T>(np);
  int32_t* scan_tmp = reinterpret_cast<int32_t*>(W.take<char>(scan_workspace(np)));
  const bool vec = al16(ci) && al16(cj) && al16(ck) && al16(vals);
  const unsigned hgrid = (unsigned)((np + kBlock / kWave - 1) / (kBlock / kWave));
  if (vec) hipLaunchKernelGGL(ttv_piece_heads_kernel<true>, dim3(hgrid), dim3(kBlock), 0, s, nnz, np, ci, cj, heads);
  else hipLaunchKernelGGL(ttv_piece_heads_kernel<false>, dim3(hgrid), dim3(kBlock), 0, s, nnz, np, ci, cj, heads);
  SPT_CHECK_LAUNCH("ttv piece heads");
  spt_status st = device_scan_i32<false>(heads, off, np, scan_tmp, s);
  if (st != SPT_OK) return st;
  const int cached = (int)std::min<int64_t>(K, kCooCacheBytes / sizeof(T));
  const bool all = cached == K;
  const unsigned grid = (unsigned)std::min<int64_t>(compute_units(), (np + kBigWaves - 1) / kBigWaves);
#define SPT_TTV_COO(VEC_, ALL_)                                                                                  \
  hipLaunchKernelGGL((ttv_coo_wave_kernel<T, VEC_, ALL_>), dim3(grid), dim3(kBig), 0, s, nnz, np, ci, cj, ck, vals, \
                     c, cached, off, out_i, out_j, out_v, out_nnz, ckey, cval)
  if (vec && all) SPT_TTV_COO(true, true);
  else if (vec) SPT_TTV_COO(true, false);
  else if (all) SPT_TTV_COO(false, true);
  else SPT_TTV_COO(false, false);
#undef SPT_TTV_COO
  SPT_CHECK_LAUNCH("ttv coo wave");
  hipLaunchKernelGGL(carry_fixup_kernel<T>, dim3((np + kBlock - 1) / kBlock), dim3(kBlock), 0, s, np, ckey, cval,
                     out_v, nullptr, 0);
  SPT_CHECK_LAUNCH("ttv carry_fixup");
  return SPT_OK;
}

template <typename T>
spt_status ttv_csf_wave(int64_t nnz64, int64_t nfib, int64_t K, const int32_t* pos, const int32_t* ck,
                        const T* vals, const T* c, T* out_v, int64_t* out_count, void* ws, size_t ws_bytes,
                        hipStream_t s) {
  const int nnz = (int)nnz64;
  const int np = (int)pieces_of(nnz64);
  if (nfib + 1 >= INT32_MAX) return fail(SPT_ERR_UNSUPPORTED, "ttv: more than 2^31 fibres");
  if (!ws || ws_bytes < ttv_csf_wave_workspace(nnz64))
    return fail(SPT_ERR_WORKSPACE, "ttv: workspace of %zu bytes needed, %zu given", ttv_csf_wave_workspace(nnz64),
                ws_bytes);
  Workspace W(ws, ws_bytes);
  int32_t* first = W.take<int32_t>(np + 1);
  int32_t* ckey = W.take<int32_t>(np);
  T* cval = W.take<T>(np);
  hipLaunchKernelGGL(ttv_piece_fibres_kernel, dim3((np + 1 + kBlock - 1) / kBlock), dim3(kBlock), 0, s, np, (int)nfib,
                     pos, first, out_count);
  SPT_CHECK_LAUNCH("ttv piece fibres");
  const bool vec = al16(ck) && al16(vals);
  const int cached = (int)std::min<int64_t>(K, kCsfCacheBytes / sizeof(T));
  const bool all = cached == K;
  const unsigned grid = (unsigned)std::min<int64_t>(compute_units(), (np + kBigWaves - 1) / kBigWaves);
#define SPT_TTV_CSF(VEC_, ALL_)                                                                                   \
  hipLaunchKernelGGL((ttv_csf_wave_kernel<T, VEC_, ALL_>), dim3(grid), dim3(kBig), 0, s, nnz, np, first, pos, ck, \
                     vals, c, cached, out_v, ckey, cval)
  if (vec && all) SPT_TTV_CSF(true, true);
  else if (vec) SPT_TTV_CSF(true, false);
  else if (all) SPT_TTV_CSF(false, true);
  else SPT_TTV_CSF(false, false);
#undef SPT_TTV_CSF
  SPT_CHECK_LAUNCH("ttv csf wave");
  hipLaunchKernelGGL(carry_fixup_kernel<T>, dim3((np + kBlock - 1) / kBlock), dim3(kBlock), 0, s, np, ckey, cval,
                     out_v, nullptr, 0);
  SPT_CHECK_LAUNCH("ttv carry_fixup");
  return SPT_OK;
}

template spt_status ttv_coo_wave<float>(int64_t, int64_t, const int32_t*, const int32_t*, const int32_t*,
                                        const float*, const float*, int32_t*, int32_t*, float*, int64_t*, void*,
                                        size_t, hipStream_t);
template spt_status ttv_coo_wave<double>(int64_t, int64_t, const int32_t*, const int32_t*, const int32_t*,
                                         const double*, const double*, int32_t*, int32_t*, double*, int64_t*, void*,
                                         size_t, hipStream_t);
template spt_status ttv_csf_wave<float>(int64_t, int64_t, int64_t, const int32_t*, const int32_t*, const float*,
                                        const float*, float*, int64_t*, void*, size_t, hipStream_t);
template spt_status ttv_csf_wave<double>(int64_t, int64_t, int64_t, const int32_t*, const int32_t*, const double*,
                                         const double*, double*, int64_t*, void*, size_t, hipStream_t);

}  // namespace spt
