// 3rd-order kernels (paper Section 5.3): TTV A_ij = sum_k B_ijk c_k and
// MTTKRP A_ij = sum_kl B_ikl C_kj D_lj on ordered COO and on CSF, gfx950.
//
// Both reduce runs of consecutive stored entries that share leading
// coordinates -- the GPU form of the paper's deduplication / iterator chaining
// over ordered non-unique levels (Section 4.3): (i,j) fibers for TTV, i slices
// for MTTKRP. Work is split evenly over stored entries; a run cut by a split
// leaves a carry that a follow-up kernel adds in a fixed order (no atomics).
#include <algorithm>

#include "common.hpp"
#include "scan.hpp"
#include "segreduce.hpp"

namespace spt {

spt_status csr_rows_reduce(int dtype, int64_t nnz, int64_t nrows, const int32_t* pos,
                           const int32_t* crd, const void* vals, const void* x, void* out,
                           void* ws, size_t ws_bytes, hipStream_t s);
size_t seg_spmv_workspace(int64_t nnz);

template <typename T>
__device__ __forceinline__ T ldg_stream(const T* p) {
  return __builtin_nontemporal_load(p);
}

template <typename T>
__global__ __launch_bounds__(kBlock) void fill_t_kernel(T* __restrict__ out, int64_t n, T value) {
  int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (i < n) out[i] = value;
}

// ================================================================ TTV on COO

constexpr int kTtvIPT = 8;
constexpr int kTtvChunk = kTtvIPT * kBlock;

__device__ __forceinline__ int ttv_slot(int e) { return e + e / kTtvIPT; }

// heads[w] = number of (i,j) fiber starts among the entries of chunk w.
// VEC: 16-byte coordinate loads (needs 16-byte aligned ci, cj).
template <bool VEC>
__global__ __launch_bounds__(kBlock) void ttv_count_kernel(int nnz, const int32_t* __restrict__ ci,
                                                           const int32_t* __restrict__ cj,
                                                           int32_t* __restrict__ heads) {
  const int base = blockIdx.x * kTtvChunk;
  int cnt = 0;
  if (VEC) {
    typedef int32_t i4 __attribute__((ext_vector_type(4)));
#pragma unroll
    for (int q = 0; q < kTtvIPT / 4; ++q) {
      const int p0 = base + (q * kBlock + threadIdx.x) * 4;
      if (p0 + 4 <= nnz) {
        const i4 a = ldg_stream(reinterpret_cast<const i4*>(ci + p0));
        const i4 b = ldg_stream(reinterpret_cast<const i4*>(cj + p0));
        int pa = -1, pb = -1;
        if (p0 > 0) {
          pa = ci[p0 - 1];
          pb = cj[p0 - 1];
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          cnt += (a[r] != pa || b[r] != pb) ? 1 : 0;
          pa = a[r];
          pb = b[r];
        }
      } else {
        for (int p = p0; p < nnz && p < p0 + 4; ++p)
          cnt += (p == 0 || ci[p] != ci[p - 1] || cj[p] != cj[p - 1]) ? 1 : 0;
      }
    }
  } else {
#pragma unroll
    for (int k = 0; k < kTtvIPT; ++k) {
      const int p = base + k * kBlock + threadIdx.x;
      if (p < nnz) cnt += (p == 0 || ci[p] != ci[p - 1] || cj[p] != cj[p - 1]) ? 1 : 0;
    }
  }
  int total;
  block_inclusive_sum(cnt, &total);
  if (threadIdx.x == 0) heads[blockIdx.x] = total;
}

__global__ void ttv_total_kernel(int nchunks, const int32_t* __restrict__ heads,
                                 const int32_t* __restrict__ off, int64_t* __restrict__ out_nnz) {
  if (threadIdx.x == 0 && blockIdx.x == 0)
    *out_nnz = nchunks > 0 ? (int64_t)off[nchunks - 1] + heads[nchunks - 1] : 0;
}

// One output entry per fiber, at index off[chunk] + rank of the fiber's head
// inside the chunk (append order = ascending (i,j), Section 3.4). The thread
// holding a head appends the coordinates; the thread holding the fiber's end
// stores the value. Carry protocol as in the SpMV kernel, keyed by output index.
template <typename T> struct TtvVec;
template <> struct TtvVec<double> { static constexpr int R = 2; typedef double type __attribute__((ext_vector_type(2))); typedef int32_t itype __attribute__((ext_vector_type(2))); };
template <> struct TtvVec<float> { static constexpr int R = 4; typedef float type __attribute__((ext_vector_type(4))); typedef int32_t itype __attribute__((ext_vector_type(4))); };

template <typename T, bool VEC>
__global__ __launch_bounds__(kBlock) void ttv_coo_kernel(
    int nnz, const int32_t* __restrict__ ci, const int32_t* __restrict__ cj,
    const int32_t* __restrict__ ck, const T* __restrict__ vals, const T* __restrict__ c,
    const int32_t* __restrict__ chunk_off, int32_t* __restrict__ out_i, int32_t* __restrict__ out_j,
    T* __restrict__ out_v, int32_t* __restrict__ carry_key, T* __restrict__ carry_val) {
  __shared__ T s_val[kTtvChunk + kBlock];
  __shared__ int32_t s_i[kTtvChunk + kBlock];
  __shared__ int32_t s_j[kTtvChunk + kBlock];
  __shared__ SegScanStorage<T> s_scan;

  const int tid = threadIdx.x;
  const int chunk = blockIdx.x;  // plain order: one sequential stream per array reads fastest
  const int base = chunk * kTtvChunk;
  const int end = min(base + kTtvChunk, nnz);
  const int32_t fill_i = ci[end - 1], fill_j = cj[end - 1];
  constexpr int R = TtvVec<T>::R;
  using V = typename TtvVec<T>::type;
  using IV = typename TtvVec<T>::itype;
#pragma unroll
  for (int q = 0; q < kTtvIPT / R; ++q) {
    const int e0 = (q * kBlock + tid) * R;
    const int p0 = base + e0;
    int32_t i[R], j[R], k[R];
    T v[R];
    bool ok[R];
    if (VEC && p0 + R <= end) {
      const IV iv = ldg_stream(reinterpret_cast<const IV*>(ci + p0));
      const IV jv = ldg_stream(reinterpret_cast<const IV*>(cj + p0));
      const IV kv = ldg_stream(reinterpret_cast<const IV*>(ck + p0));
      const V vv = ldg_stream(reinterpret_cast<const V*>(vals + p0));
#pragma unroll
      for (int r = 0; r < R; ++r) {
        i[r] = iv[r];
        j[r] = jv[r];
        k[r] = kv[r];
        v[r] = vv[r];
        ok[r] = true;
      }
    } else {
#pragma unroll
      for (int r = 0; r < R; ++r) {
        ok[r] = p0 + r < end;
        i[r] = ok[r] ? ldg_stream(ci + p0 + r) : fill_i;
        j[r] = ok[r] ? ldg_stream(cj + p0 + r) : fill_j;
        k[r] = ok[r] ? ldg_stream(ck + p0 + r) : 0;
        v[r] = ok[r] ? ldg_stream(vals + p0 + r) : T(0);
      }
    }
#pragma unroll
    for (int r = 0; r < R; ++r) {
      s_val[ttv_slot(e0 + r)] = ok[r] ? v[r] * c[k[r]] : T(0);
      s_i[ttv_slot(e0 + r)] = i[r];
      s_j[ttv_slot(e0 + r)] = j[r];
    }
  }
  int32_t pi = -1, pj = -1;  // coordinates of the entry before this thread's items
  if (tid == 0 && base > 0) {
    pi = ci[base - 1];
    pj = cj[base - 1];
  }
  __syncthreads();
  if (tid > 0) {
    pi = s_i[ttv_slot(tid * kTtvIPT - 1)];
    pj = s_j[ttv_slot(tid * kTtvIPT - 1)];
  }

  int32_t li[kTtvIPT], lj[kTtvIPT];
  unsigned headmask = 0;
  {
    int32_t qi = pi, qj = pj;
#pragma unroll
    for (int k = 0; k < kTtvIPT; ++k) {
      li[k] = s_i[ttv_slot(tid * kTtvIPT + k)];
      lj[k] = s_j[ttv_slot(tid * kTtvIPT + k)];
      if (li[k] != qi || lj[k] != qj) headmask |= 1u << k;
      qi = li[k];
      qj = lj[k];
    }
  }
  const int cnt = __popc(headmask);
  int wg_heads;
  int next_idx = chunk_off[chunk] + block_inclusive_sum(cnt, &wg_heads) - cnt;

  T acc = 0, lead = 0;
  int has_head = 0, last_key = -1;
#pragma unroll
  for (int k = 0; k < kTtvIPT; ++k) {
    if (headmask & (1u << k)) {
      if (!has_head) {
        lead = acc;
        has_head = 1;
      } else {
        out_v[last_key] = acc;
      }
      last_key = next_idx++;
      out_i[last_key] = li[k];
      out_j[last_key] = lj[k];
      acc = 0;
    }
    acc += s_val[ttv_slot(tid * kTtvIPT + k)];
  }

  SegSum<T> in = block_seg_exclusive_scan<T>(SegSum<T>{has_head, acc, last_key}, s_scan);
  const int carry_idx = chunk_off[chunk] - 1;  // fiber cut by the chunk start
  if (has_head) {
    const T total = in.v + lead;
    if (in.f) {
      out_v[in.k] = total;
    } else {
      const bool at_start = (tid == 0) && (headmask & 1u);
      carry_key[chunk] = at_start ? -1 : carry_idx;
      carry_val[chunk] = total;
    }
  }
  if (tid == kBlock - 1) {
    if (has_head) {
      out_v[last_key] = acc;
    } else if (in.f) {
      out_v[in.k] = in.v + acc;
    } else {
      carry_key[chunk] = carry_idx;
      carry_val[chunk] = in.v + acc;
    }
  }
}

static size_t ttv_coo_workspace(int64_t nnz) {
  const int64_t nch = (nnz + kTtvChunk - 1) / kTtvChunk;
  return 3 * align_up((size_t)nch * 4, 256) + align_up((size_t)nch * 8, 256) + scan_workspace(nch) +
         256;
}

template <typename T>
static spt_status ttv_coo_typed(const spt_tensor* B, const T* c, int32_t* out_i, int32_t* out_j,
                                T* out_v, int64_t* out_nnz, void* ws, size_t ws_bytes,
                                hipStream_t s) {
  const int64_t nnz64 = B->nvals;
  if (nnz64 + kTtvChunk >= INT32_MAX) return fail(SPT_ERR_UNSUPPORTED, "ttv: more than 2^31 entries");
  const int nnz = (int)nnz64;
  const int nch = (nnz + kTtvChunk - 1) / kTtvChunk;
  if (nnz == 0) {
    hipLaunchKernelGGL(ttv_total_kernel, dim3(1), dim3(kWave), 0, s, 0, nullptr, nullptr, out_nnz);
    SPT_CHECK_LAUNCH("ttv_total");
    return SPT_OK;
  }
  if (!ws || ws_bytes < ttv_coo_workspace(nnz))
    return fail(SPT_ERR_WORKSPACE, "ttv: workspace of %zu bytes needed, %zu given",
                ttv_coo_workspace(nnz), ws_bytes);
  Workspace W(ws, ws_bytes);
  int32_t* heads = W.take<int32_t>(nch);
  int32_t* off = W.take<int32_t>(nch);
  int32_t* ckey = W.take<int32_t>(nch);
  T* cval = W.take<T>(nch);
  int32_t* scan_tmp = reinterpret_cast<int32_t*>(W.take<char>(scan_workspace(nch)));
  const int32_t *ci = B->level[0].crd, *cj = B->level[1].crd, *ck = B->level[2].crd;
  auto al = [](const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; };
  const bool vec = al(ci) && al(cj) && al(ck) && al(B->vals);
  if (vec) hipLaunchKernelGGL(ttv_count_kernel<true>, dim3(nch), dim3(kBlock), 0, s, nnz, ci, cj, heads);
  else hipLaunchKernelGGL(ttv_count_kernel<false>, dim3(nch), dim3(kBlock), 0, s, nnz, ci, cj, heads);
  SPT_CHECK_LAUNCH("ttv_count");
  spt_status st = device_scan_i32<false>(heads, off, nch, scan_tmp, s);
  if (st != SPT_OK) return st;
  hipLaunchKernelGGL(ttv_total_kernel, dim3(1), dim3(kWave), 0, s, nch, heads, off, out_nnz);
  SPT_CHECK_LAUNCH("ttv_total");
  if (vec)
    hipLaunchKernelGGL((ttv_coo_kernel<T, true>), dim3(nch), dim3(kBlock), 0, s, nnz, ci, cj, ck,
                       static_cast<const T*>(B->vals), c, off, out_i, out_j, out_v, ckey, cval);
  else
    hipLaunchKernelGGL((ttv_coo_kernel<T, false>), dim3(nch), dim3(kBlock), 0, s, nnz, ci, cj, ck,
                       static_cast<const T*>(B->vals), c, off, out_i, out_j, out_v, ckey, cval);
  SPT_CHECK_LAUNCH("ttv_coo");
  hipLaunchKernelGGL(carry_fixup_kernel<T>, dim3((nch + kBlock - 1) / kBlock), dim3(kBlock), 0, s,
                     nch, ckey, cval, out_v);
  SPT_CHECK_LAUNCH("ttv carry_fixup");
  return SPT_OK;
}

// ================================================================ MTTKRP
//
// G lanes (32 or 64) work on one stored entry at a time, lane gl owning output
// column jt*G + gl; a workgroup has 256/G such groups, each walking kEPG
// consecutive entries and keeping the running row sum in a register. Entry
// coordinates are loaded G at a time (coalesced) and broadcast with shuffles;
// the factor rows C[k,:], D[l,:] are gathered as contiguous G-wide rows.
// LEVEL2 = the same reduction applied to the (key, vector) carries of level 1.
// CSF    = i and k come from the upper levels (expanded into LDS per chunk) and
//          the product with C[k,:] is applied once per fiber piece (factored
//          form, Section 5.3 / CSF being the more efficient format).
// entries walked by one group of lanes, per mode: the CSF pre-phase is amortised over a
// longer walk; the carry level is small and wants parallelism instead
enum { MT_COO = 0, MT_LEVEL2 = 1, MT_CSF = 2, MT_SPDM = 3 };
template <int MODE> struct Epg { static constexpr int value = MODE == 2 ? 256 : (MODE == 1 ? 32 : 128); };
constexpr int kU = 8;  // entries whose factor rows are in flight together

template <typename T, int G>
struct MttkrpShared {
  T lead[kBlock / G][G];
  T tail[kBlock / G][G];
  int has_head[kBlock / G];
  int first_close[kBlock / G];
  int last_key[kBlock / G];
  int empty[kBlock / G];
};


// First r in [0, n] with a[r] >= target (a ascending, n entries).
__device__ __forceinline__ int first_at_or_after(const int32_t* __restrict__ a, int n, int target) {
  int lo = 0, hi = n;
  while (lo < hi) {
    const int mid = lo + ((hi - lo) >> 1);
    if (a[mid] < target) lo = mid + 1; else hi = mid;
  }
  return lo;
}

// CSF: for chunk boundary c (entries from c * chunk on), out[3c] = first fiber that starts at or
// after it, out[3c+1] = first slice that starts at or after that fiber, out[3c+2] = the same as
// the end of the chunk before (all slices once the fibers are used up). Boundary nchunks = the end.
__global__ __launch_bounds__(kBlock) void csf_chunk_bounds_kernel(
    int nchunks, int chunk, int nslices, int nfibers, const int32_t* __restrict__ pos1,
    const int32_t* __restrict__ pos2, int32_t* __restrict__ out) {
  const int c = blockIdx.x * kBlock + threadIdx.x;
  if (c > nchunks) return;
  const int f = c == nchunks ? nfibers : first_at_or_after(pos2, nfibers + 1, c * chunk);
  const int sl = first_at_or_after(pos1, nslices + 1, f);
  out[3 * c] = f;
  out[3 * c + 1] = sl;
  out[3 * c + 2] = f >= nfibers ? nslices : sl;
}

// Broadcast of lane (addr / 4)'s value through the LDS crossbar.
__device__ __forceinline__ int32_t bperm(int addr, int32_t v) { return __builtin_amdgcn_ds_bpermute(addr, v); }
__device__ __forceinline__ float bperm(int addr, float v) {
  return __int_as_float(__builtin_amdgcn_ds_bpermute(addr, __float_as_int(v)));
}
__device__ __forceinline__ double bperm(int addr, double v) {
  const int lo = __builtin_amdgcn_ds_bpermute(addr, __double2loint(v));
  const int hi = __builtin_amdgcn_ds_bpermute(addr, __double2hiint(v));
  return __hiloint2double(hi, lo);
}

// FAST: the factor matrices are addressed with 32-bit byte offsets formed by one 24-bit
// multiply-add (host-checked: dimensions and J * sizeof(T) below 2^23, matrices below 4 GiB),
// and no load of the batch sits behind a branch: a batch slot beyond the group's entries
// repeats the last entry, a lane beyond column J reads column J - 1 (neither is ever stored).
// The 64-bit multiply-adds and the per-entry branches of the general path cost more vector
// instructions than the arithmetic itself.
template <typename T, int G, int MODE, bool FAST>
__global__ __launch_bounds__(kBlock) void mttkrp_kernel(
    int n, int J,
    // COO: ci/ck/cl; CSF: cl only (crd of level 2) plus the upper levels below
    const int32_t* __restrict__ ci, const int32_t* __restrict__ ck, const int32_t* __restrict__ cl,
    const T* __restrict__ vals, const T* __restrict__ Cm, const T* __restrict__ Dm,
    // CSF upper levels
    const int32_t* __restrict__ crd0, const int32_t* __restrict__ pos1, const int32_t* __restrict__ crd1,
    const int32_t* __restrict__ pos2, int nslices, int nfibers,
    // LEVEL2 input
    const int32_t* __restrict__ in_key, const T* __restrict__ in_vec,
    T* __restrict__ A, int32_t* __restrict__ carry_key, T* __restrict__ carry_vec) {
  constexpr int NG = kBlock / G;
  constexpr int kEPG = Epg<MODE>::value;
  constexpr int CHUNK = NG * kEPG;
  __shared__ MttkrpShared<T, G> sh;
  __shared__ int32_t s_i[MODE == MT_CSF ? CHUNK : 1];
  __shared__ int32_t s_k[MODE == MT_CSF ? CHUNK : 1];
  __shared__ int s_mark0;
  // SpDM closes a row every few entries. A store issued between two batches of gathers
  // makes the next batch wait for the store's acknowledgement (loads and stores retire
  // through one counter), so closed rows are parked in LDS and written out in bursts.
  constexpr int kRowBuf = 16;
  __shared__ T s_rowv[MODE == MT_SPDM ? NG : 1][MODE == MT_SPDM ? kRowBuf : 1][G];
  __shared__ int s_rowk[MODE == MT_SPDM ? NG : 1][MODE == MT_SPDM ? kRowBuf : 1];
  int nbuf = 0;

  const int tid = threadIdx.x;
  const int g = tid / G, gl = tid % G;
  const int j = blockIdx.y * G + gl;
  const bool jok = j < J;
  // FAST: byte address of lane 0 of this lane's group for the broadcasts, bytes per factor
  // row and this lane's byte offset inside a row
  const int half_base = 4 * (lane_id() & ~(G - 1));
  const uint32_t jbytes = static_cast<uint32_t>(J) * sizeof(T);
  const uint32_t joff = static_cast<uint32_t>(min(j, J - 1)) * sizeof(T);
  const int chunk = xcd_contiguous_block_id();
  const int chunk_base = chunk * CHUNK;
  const int chunk_end = min(chunk_base + CHUNK, n);

  if (MODE == MT_CSF) {
    // Expand the coordinates of levels 0 and 1 for the entries of this chunk:
    // mark the first entry of every fiber / slice that starts inside the chunk,
    // then let every entry take the last mark at or before it.
    // fibers [f_lo, f_hi) and slices [s_lo, s_hi) start inside the chunk; found beforehand, one
    // bisection per chunk boundary (csf_chunk_bounds_kernel), passed through in_key
    const int f_lo = in_key[3 * chunk], f_hi = in_key[3 * chunk + 3];
    for (int e = tid; e < CHUNK; e += kBlock) {
      s_i[e] = -1;
      s_k[e] = -1;
    }
    __syncthreads();
    for (int f = f_lo + tid; f < f_hi; f += kBlock) {
      const int a = pos2[f];
      if (pos2[f + 1] > a) s_k[a - chunk_base] = crd1[f];
    }
    __syncthreads();
    const int s_lo = in_key[3 * chunk + 1], s_hi = in_key[3 * chunk + 5];
    // a slice is marked at its first stored entry, whichever of its fibers holds it (a
    // compressed level may hold empty segments: leading fibers of a slice can be empty)
    for (int sl = s_lo + tid; sl < s_hi; sl += kBlock) {
      const int a = pos2[pos1[sl]];
      if (pos2[pos1[sl + 1]] > a && a < chunk_base + CHUNK) s_i[a - chunk_base] = crd0[sl];
    }
    __syncthreads();
    // propagate marks forward: 256 threads, CHUNK/256 consecutive entries each
    constexpr int PER = CHUNK / kBlock;
    int li = -1, lk = -1;
    if (tid == 0) s_mark0 = s_i[0] >= 0;  // the chunk starts on a slice head
#pragma unroll
    for (int q = 0; q < PER; ++q) {
      const int e = tid * PER + q;
      if (s_i[e] >= 0) li = s_i[e];
      if (s_k[e] >= 0) lk = s_k[e];
    }
    // exclusive "last mark" over threads; reuse the segmented scan's key lane
    __shared__ SegScanStorage<int> s_sc;
    SegSum<int> a = block_seg_exclusive_scan<int>(SegSum<int>{li >= 0, 0, li}, s_sc);
    __syncthreads();
    SegSum<int> b = block_seg_exclusive_scan<int>(SegSum<int>{lk >= 0, 0, lk}, s_sc);
    // carry-in coordinates of the chunk: the slice / fiber cut by its start
    int run_i = a.f ? a.k : (s_lo > 0 ? crd0[s_lo - 1] : -1);
    int run_k = b.f ? b.k : (f_lo > 0 ? crd1[f_lo - 1] : -1);
#pragma unroll
    for (int q = 0; q < PER; ++q) {
      const int e = tid * PER + q;
      if (s_i[e] >= 0) run_i = s_i[e];
      else s_i[e] = run_i;
      if (s_k[e] >= 0) run_k = s_k[e];
      else s_k[e] = run_k;
    }
    __syncthreads();
  }

  // ---- group walk
  const int g0 = chunk_base + g * kEPG;
  const int g1 = min(g0 + kEPG, chunk_end);
  T acc = 0, lead = 0, t = 0, c_cur = 0;
  int has_head = 0, first_close = -1;
  int cur = -1, cur_k = -1;
  // cur = slice coordinate of the entry just before this group's first entry
  // (-1: there is none; -2: unknown but different, the group starts on a head)
  if (g0 < g1) {
    if (MODE == MT_COO || MODE == MT_SPDM) cur = g0 > 0 ? ci[g0 - 1] : -1;
    if (MODE == MT_LEVEL2) cur = g0 > 0 ? in_key[g0 - 1] : -1;
    if (MODE == MT_CSF) {
      if (g0 > chunk_base) cur = s_i[g0 - 1 - chunk_base];
      else cur = chunk_base == 0 ? -1 : (s_mark0 ? -2 : s_i[0]);
    }
  }

  for (int b0 = g0; b0 < g1; b0 += G) {
    const int p_l = b0 + gl;
    int32_t ri = 0, rk = 0, rl = 0;
    T rv = 0;
    if (p_l < g1) {
      if (MODE == MT_COO || MODE == MT_SPDM) {
        ri = ldg_stream(ci + p_l);
        rk = ldg_stream(ck + p_l);
        if (MODE == MT_COO) rl = ldg_stream(cl + p_l);
        rv = ldg_stream(vals + p_l);
      } else if (MODE == MT_CSF) {
        ri = s_i[p_l - chunk_base];
        rk = s_k[p_l - chunk_base];
        rl = ldg_stream(cl + p_l);
        rv = ldg_stream(vals + p_l);
      } else {
        ri = in_key[p_l];
      }
    }
    const int cntb = min(G, g1 - b0);
    // kU entries at a time: first issue all their factor-row loads (they are
    // independent, so the cache latency is paid once per batch, not per entry),
    // then run the segment logic over the batch in order.
    for (int s0 = 0; s0 < cntb; s0 += kU) {
      int ii[kU];
      T fa[kU], fb[kU], vv[kU];
      bool fh[kU];
      int pi = cur, pk = cur_k;
#pragma unroll
      for (int u = 0; u < kU; ++u) {
        const int sidx = s0 + u;  // < G because kU divides G
        const bool live = sidx < cntb;
        fh[u] = false;
        vv[u] = T(1);
        fb[u] = T(1);
        if (FAST && MODE != MT_LEVEL2) {
          const int addr = half_base + 4 * min(sidx, cntb - 1);
          ii[u] = bperm(addr, ri);
          const int k = bperm(addr, rk);
          vv[u] = bperm(addr, rv);
          const int l = MODE != MT_SPDM ? bperm(addr, rl) : 0;
          fa[u] = *reinterpret_cast<const T*>(reinterpret_cast<const char*>(Cm) + (__umul24(k, jbytes) + joff));
          if (MODE != MT_SPDM)
            fb[u] = *reinterpret_cast<const T*>(reinterpret_cast<const char*>(Dm) + (__umul24(l, jbytes) + joff));
          if (MODE == MT_CSF) {  // C[k,:] is used where a new (i,k) fiber piece starts
            fh[u] = live && (ii[u] != pi || k != pk);
            if (live) {
              pi = ii[u];
              pk = k;
            }
          }
          continue;
        }
        ii[u] = __shfl(ri, sidx, G);
        if (MODE == MT_LEVEL2) {
          fa[u] = (live && jok) ? in_vec[(int64_t)(b0 + sidx) * J + j] : T(0);
        } else {
          const int k = __shfl(rk, sidx, G);
          const int l = __shfl(rl, sidx, G);
          vv[u] = __shfl(rv, sidx, G);
          if (MODE != MT_SPDM) fb[u] = (live && jok) ? Dm[(int64_t)l * J + j] : T(0);
          if (MODE == MT_COO || MODE == MT_SPDM) {
            fa[u] = (live && jok) ? Cm[(int64_t)k * J + j] : T(0);
          } else {  // CSF: C[k,:] only where a new (i,k) fiber piece starts
            fh[u] = live && (ii[u] != pi || k != pk);
            fa[u] = (fh[u] && jok) ? Cm[(int64_t)k * J + j] : T(0);
            if (live) {
              pi = ii[u];
              pk = k;
            }
          }
        }
      }
      cur_k = pk;
#pragma unroll
      for (int u = 0; u < kU; ++u) {
        if (s0 + u < cntb) {
          const int i = ii[u];
          if (MODE == MT_CSF && fh[u]) {  // factored form: close the previous fiber piece
            acc += c_cur * t;
            t = 0;
            c_cur = fa[u];
          }
          if (i != cur) {
            if (!has_head) {
              lead = acc;
              has_head = 1;
              first_close = cur;
            } else if (cur >= 0) {
              if (MODE == MT_SPDM) {
                s_rowv[g][nbuf][gl] = acc;
                if (gl == 0) s_rowk[g][nbuf] = cur;
                ++nbuf;
              } else if (jok) {
                if (MODE == MT_LEVEL2) A[(int64_t)cur * J + j] += acc;
                else A[(int64_t)cur * J + j] = acc;
              }
            }
            acc = 0;
            cur = i;
          }
          if (MODE == MT_CSF) t += vv[u] * fb[u];
          else if (MODE == MT_COO) acc += vv[u] * fa[u] * fb[u];
          else if (MODE == MT_SPDM) acc += vv[u] * fa[u];
          else acc += fa[u];
        }
      }
      if (MODE == MT_SPDM && nbuf > kRowBuf - kU) {
        for (int r = 0; r < nbuf; ++r)
          if (jok) __builtin_nontemporal_store(s_rowv[g][r][gl], &A[(int64_t)s_rowk[g][r] * J + j]);
        nbuf = 0;
      }
    }
  }
  if (MODE == MT_SPDM) {
    for (int r = 0; r < nbuf; ++r)
      if (jok) __builtin_nontemporal_store(s_rowv[g][r][gl], &A[(int64_t)s_rowk[g][r] * J + j]);
  }
  if (MODE == MT_CSF) acc += c_cur * t;

  sh.lead[g][gl] = lead;
  sh.tail[g][gl] = acc;
  if (gl == 0) {
    sh.has_head[g] = has_head;
    sh.first_close[g] = first_close;
    sh.last_key[g] = cur;
    sh.empty[g] = g0 >= g1;
  }
  __syncthreads();

  // ---- resolve the NG group summaries in order (threads of group 0)
  if (g == 0) {
    T run = 0;
    bool seen = false, carried = false;
    int last = -1;
    for (int q = 0; q < NG; ++q) {
      if (sh.empty[q]) continue;
      if (sh.has_head[q]) {
        const T total = run + sh.lead[q][gl];
        const int key = sh.first_close[q];
        if (seen) {
          if (jok && key >= 0) {
            if (MODE == MT_LEVEL2) A[(int64_t)key * J + j] += total;
            else A[(int64_t)key * J + j] = total;
          }
        } else {  // precedes the first head of the chunk: carry (key < 0: nothing precedes)
          if (jok) carry_vec[(int64_t)chunk * J + j] = total;
          if (gl == 0 && blockIdx.y == 0) carry_key[chunk] = key < 0 ? -1 : key;
          carried = true;
        }
        run = sh.tail[q][gl];
        seen = true;
      } else {
        run += sh.tail[q][gl];
      }
      last = sh.last_key[q];
    }
    if (seen) {
      if (jok && last >= 0) {
        if (MODE == MT_LEVEL2) A[(int64_t)last * J + j] += run;
        else A[(int64_t)last * J + j] = run;
      }
    } else if (!carried) {
      if (jok) carry_vec[(int64_t)chunk * J + j] = run;
      if (gl == 0 && blockIdx.y == 0) carry_key[chunk] = last;
    }
  }
}

// Adds the remaining (key, vector) carries into A, one thread per (carry, j);
// the thread at the start of a run of equal keys adds the whole run in order.
template <typename T>
__global__ __launch_bounds__(kBlock) void vec_carry_fixup_kernel(int n, int J,
                                                                 const int32_t* __restrict__ key,
                                                                 const T* __restrict__ vec,
                                                                 T* __restrict__ A) {
  const int64_t idx = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (idx >= (int64_t)n * J) return;
  const int w = (int)(idx / J), j = (int)(idx % J);
  const int32_t kk = key[w];
  if (kk < 0) return;
  if (w > 0 && key[w - 1] == kk) return;
  double s = 0;
  for (int u = w; u < n && key[u] == kk; ++u) s += (double)vec[(int64_t)u * J + j];
  A[(int64_t)kk * J + j] = (T)((double)A[(int64_t)kk * J + j] + s);
}

static int mttkrp_group(int J) { return J <= 32 ? 32 : 64; }
static int mttkrp_chunk(int J, int mode) {
  const int epg = mode == MT_CSF ? Epg<MT_CSF>::value : (mode == MT_LEVEL2 ? Epg<MT_LEVEL2>::value : Epg<MT_COO>::value);
  return (kBlock / mttkrp_group(J)) * epg;
}

size_t mttkrp_workspace(Format, const spt_tensor* B, int32_t J) {
  if (J < 1) J = 1;
  const int64_t chunk = mttkrp_chunk(J, MT_COO);  // the smaller level-1 chunk of the two formats
  const int64_t chunk2 = mttkrp_chunk(J, MT_LEVEL2);
  const int64_t n1 = (B->nvals + chunk - 1) / chunk;
  const int64_t n2 = (n1 + chunk2 - 1) / chunk2;
  return align_up((size_t)n1 * 4, 256) + align_up((size_t)n1 * J * 8, 256) +
         align_up((size_t)n2 * 4, 256) + align_up((size_t)n2 * J * 8, 256) +
         align_up((size_t)(n1 + 1) * 12, 256) + 256;
}

// rows_override / cols_override (SpDM mode only): row and column index per stored entry taken
// from these arrays instead of B's first two levels, and no zero fill of A (every output row
// then has at least one entry, and rows with entries are stored, not accumulated).
template <typename T, int G, bool FAST>
static spt_status mttkrp_launch(Format f, const spt_tensor* B, const T* Cm, const T* Dm, int J,
                                T* A, void* ws, size_t ws_bytes, hipStream_t s,
                                const int32_t* rows_override = nullptr,
                                const int32_t* cols_override = nullptr) {
  const int CHUNK = mttkrp_chunk(J, f == Format::CSF3 ? MT_CSF : MT_COO);
  const int CHUNK2 = mttkrp_chunk(J, MT_LEVEL2);
  const int64_t I = B->level[0].N;
  const int64_t nnz64 = B->nvals;
  if (nnz64 + CHUNK >= INT32_MAX || I * J >= ((int64_t)1 << 38))
    return fail(SPT_ERR_UNSUPPORTED, "mttkrp: tensor too large");
  if (I * J > 0 && !rows_override) {
    hipLaunchKernelGGL(fill_t_kernel<T>, dim3((unsigned)((I * J + kBlock - 1) / kBlock)),
                       dim3(kBlock), 0, s, A, I * J, T(0));
    SPT_CHECK_LAUNCH("mttkrp fill");
  }
  const int nnz = (int)nnz64;
  if (nnz == 0) return SPT_OK;
  if (!ws || ws_bytes < mttkrp_workspace(f, B, J))
    return fail(SPT_ERR_WORKSPACE, "mttkrp: workspace of %zu bytes needed, %zu given",
                mttkrp_workspace(f, B, J), ws_bytes);
  const int n1 = (nnz + CHUNK - 1) / CHUNK;
  const int n2 = (n1 + CHUNK2 - 1) / CHUNK2;
  Workspace W(ws, ws_bytes);
  int32_t* key1 = W.take<int32_t>(n1);
  T* vec1 = W.take<T>((size_t)n1 * J);
  int32_t* key2 = W.take<int32_t>(n2);
  T* vec2 = W.take<T>((size_t)n2 * J);
  const unsigned jt = (unsigned)((J + G - 1) / G);
  const spt_level* L = B->level;
  if (f == Format::COO2) {  // SpDM: the same slice reduction with one dense factor
    hipLaunchKernelGGL((mttkrp_kernel<T, G, MT_SPDM, FAST>), dim3(n1, jt), dim3(kBlock), 0, s, nnz, J,
                       rows_override ? rows_override : L[0].crd,
                       cols_override ? cols_override : L[1].crd, nullptr,
                       static_cast<const T*>(B->vals), Cm, nullptr, nullptr, nullptr, nullptr, nullptr,
                       0, 0, nullptr, nullptr, A, key1, vec1);
  } else if (f == Format::COO3) {
    hipLaunchKernelGGL((mttkrp_kernel<T, G, MT_COO, FAST>), dim3(n1, jt), dim3(kBlock), 0, s, nnz, J,
                       L[0].crd, L[1].crd, L[2].crd, static_cast<const T*>(B->vals), Cm, Dm, nullptr,
                       nullptr, nullptr, nullptr, 0, 0, nullptr, nullptr, A, key1, vec1);
  } else {
    const int64_t nsl = L[1].M, nfib = L[2].M;
    if (nsl + 1 >= INT32_MAX || nfib + 1 >= INT32_MAX)
      return fail(SPT_ERR_UNSUPPORTED, "mttkrp: tensor too large");
    int32_t* bounds = W.take<int32_t>(3 * ((size_t)n1 + 1));
    hipLaunchKernelGGL(csf_chunk_bounds_kernel, dim3((n1 + 1 + kBlock - 1) / kBlock), dim3(kBlock), 0, s,
                       n1, CHUNK, (int)nsl, (int)nfib, L[1].pos, L[2].pos, bounds);
    SPT_CHECK_LAUNCH("csf chunk bounds");
    hipLaunchKernelGGL((mttkrp_kernel<T, G, MT_CSF, FAST>), dim3(n1, jt), dim3(kBlock), 0, s, nnz, J,
                       nullptr, nullptr, L[2].crd, static_cast<const T*>(B->vals), Cm, Dm, L[0].crd,
                       L[1].pos, L[1].crd, L[2].pos, (int)nsl, (int)nfib, bounds, nullptr, A, key1,
                       vec1);
  }
  SPT_CHECK_LAUNCH("mttkrp");
  hipLaunchKernelGGL((mttkrp_kernel<T, G, MT_LEVEL2, false>), dim3(n2, jt), dim3(kBlock), 0, s, n1, J,
                     nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr,
                     nullptr, 0, 0, key1, vec1, A, key2, vec2);
  SPT_CHECK_LAUNCH("mttkrp level 2");
  const int64_t tot = (int64_t)n2 * J;
  hipLaunchKernelGGL(vec_carry_fixup_kernel<T>, dim3((unsigned)((tot + kBlock - 1) / kBlock)),
                     dim3(kBlock), 0, s, n2, J, key2, vec2, A);
  SPT_CHECK_LAUNCH("mttkrp fixup");
  return SPT_OK;
}

template <typename T>
static spt_status mttkrp_typed(Format f, const spt_tensor* B, const void* C, const void* D, int J,
                               void* A, void* ws, size_t ws_bytes, hipStream_t s,
                               const int32_t* rows_override = nullptr,
                               const int32_t* cols_override = nullptr) {
  const T* Cm = static_cast<const T*>(C);
  const T* Dm = static_cast<const T*>(D);
  // 32-bit factor addressing: every coordinate and the row size below 2^23 (one 24-bit multiply),
  // every factor matrix below 4 GiB
  int64_t big = 0;  // the largest dimension bounds every coordinate that indexes a factor row
  for (int k = 0; k < B->nlevels; ++k) big = std::max(big, B->level[k].N);
  const int64_t rowb = (int64_t)J * (int64_t)sizeof(T);
  const bool fast = big < (1 << 23) && rowb < (1 << 23) && big * rowb < ((int64_t)1 << 32);
  if (mttkrp_group(J) == 32) {
    if (fast)
      return mttkrp_launch<T, 32, true>(f, B, Cm, Dm, J, static_cast<T*>(A), ws, ws_bytes, s, rows_override,
                                        cols_override);
    return mttkrp_launch<T, 32, false>(f, B, Cm, Dm, J, static_cast<T*>(A), ws, ws_bytes, s, rows_override,
                                       cols_override);
  }
  if (fast)
    return mttkrp_launch<T, 64, true>(f, B, Cm, Dm, J, static_cast<T*>(A), ws, ws_bytes, s, rows_override,
                                      cols_override);
  return mttkrp_launch<T, 64, false>(f, B, Cm, Dm, J, static_cast<T*>(A), ws, ws_bytes, s, rows_override,
                                     cols_override);
}

// SpDM A = B C (Section 5.2, Figure 11): B an ordered COO matrix, C and A dense row-major.
spt_status spdm_dispatch(const spt_tensor* B, const void* C, int32_t J, void* A_out, void* ws,
                         size_t ws_bytes, hipStream_t s) {
  if (!(B->level[0].flags & SPT_ORDERED))
    return fail(SPT_ERR_UNSUPPORTED, "spdm: the row level of B must be ordered");
  if (B->dtype == SPT_F64)
    return mttkrp_typed<double>(Format::COO2, B, C, nullptr, J, A_out, ws, ws_bytes, s);
  return mttkrp_typed<float>(Format::COO2, B, C, nullptr, J, A_out, ws, ws_bytes, s);
}

spt_status mttkrp_dispatch(Format f, const spt_tensor* B, const void* C, const void* D, int32_t J,
                           void* A_out, void* ws, size_t ws_bytes, hipStream_t s) {
  for (int k = 0; k < 3; ++k)
    if (!(B->level[k].flags & SPT_ORDERED))
      return fail(SPT_ERR_UNSUPPORTED, "mttkrp: every level of B must be ordered");
  if (B->dtype == SPT_F64) return mttkrp_typed<double>(f, B, C, D, J, A_out, ws, ws_bytes, s);
  return mttkrp_typed<float>(f, B, C, D, J, A_out, ws, ws_bytes, s);
}

// ================================================================ TTV dispatch

__global__ void set_i64_kernel(int64_t* out, int64_t v) {
  if (threadIdx.x == 0 && blockIdx.x == 0) *out = v;
}

// ================================================================ TTM
//
// A_ijk = sum_l B_ijl C_kl (Section 5.3): every (i,j) fibre of B yields one dense fibre of K
// values, A[f, :] = sum over the fibre's entries of B_ijl * C[:, l]. With the fibre index as
// row and l as column this is the sparse-times-dense reduction of SpDM against C transposed,
// so TTM = (fibre index per entry) + (C transposed into the workspace) + the SpDM kernels.

// COO: fid[p] = index of the (i,j) fibre of entry p; the thread holding a fibre's first
// entry appends its coordinates (append order = ascending (i,j)). Chunks as in ttv_count_kernel.
template <bool VEC>
__global__ __launch_bounds__(kBlock) void fiber_ids_kernel(int nnz, const int32_t* __restrict__ ci,
                                                           const int32_t* __restrict__ cj,
                                                           const int32_t* __restrict__ chunk_off,
                                                           int32_t* __restrict__ fid,
                                                           int32_t* __restrict__ out_i,
                                                           int32_t* __restrict__ out_j) {
  typedef int32_t i4 __attribute__((ext_vector_type(4)));
  static_assert(kTtvIPT == 8, "two 16-byte loads per array and thread");
  const int p0 = blockIdx.x * kTtvChunk + threadIdx.x * kTtvIPT;
  int32_t li[kTtvIPT], lj[kTtvIPT];
  int32_t qi = -1, qj = -1;
  if (p0 > 0 && p0 < nnz) {
    qi = ci[p0 - 1];
    qj = cj[p0 - 1];
  }
  const bool full = VEC && p0 + kTtvIPT <= nnz;
  if (full) {
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const i4 a = *reinterpret_cast<const i4*>(ci + p0 + 4 * h);
      const i4 b = *reinterpret_cast<const i4*>(cj + p0 + 4 * h);
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        li[4 * h + r] = a[r];
        lj[4 * h + r] = b[r];
      }
    }
  } else {
#pragma unroll
    for (int k = 0; k < kTtvIPT; ++k) {
      li[k] = p0 + k < nnz ? ci[p0 + k] : -1;
      lj[k] = p0 + k < nnz ? cj[p0 + k] : -1;
    }
  }
  unsigned headmask = 0;
#pragma unroll
  for (int k = 0; k < kTtvIPT; ++k) {
    if (p0 + k < nnz && (li[k] != qi || lj[k] != qj)) headmask |= 1u << k;
    qi = li[k];
    qj = lj[k];
  }
  const int cnt = __popc(headmask);
  int total;
  int running = chunk_off[blockIdx.x] + block_inclusive_sum(cnt, &total) - cnt - 1;
  int32_t lf[kTtvIPT];
#pragma unroll
  for (int k = 0; k < kTtvIPT; ++k) {
    if (headmask & (1u << k)) {
      ++running;
      out_i[running] = li[k];
      out_j[running] = lj[k];
    }
    lf[k] = running;
  }
  if (full) {
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      i4 v;
#pragma unroll
      for (int r = 0; r < 4; ++r) v[r] = lf[4 * h + r];
      *reinterpret_cast<i4*>(fid + p0 + 4 * h) = v;
    }
  } else {
#pragma unroll
    for (int k = 0; k < kTtvIPT; ++k)
      if (p0 + k < nnz) fid[p0 + k] = lf[k];
  }
}

// CSF: the fibre of entry p is the position f of level 1 with pos2[f] <= p < pos2[f+1].
__global__ __launch_bounds__(kBlock) void expand_fiber_ids_kernel(int nfib,
                                                                  const int32_t* __restrict__ pos2,
                                                                  int32_t* __restrict__ fid) {
  const int f = blockIdx.x * kBlock + threadIdx.x;
  if (f >= nfib) return;
  const int a = pos2[f], b = pos2[f + 1];
  for (int p = a; p < b; ++p) fid[p] = f;
}

// CSF: a fibre without entries (a compressed level may hold empty segments) still owns K
// output values; no entry ever writes them, so they are set to zero here. One lane per
// (fibre, k) pair would read pos2 K times: a lane tests one fibre and the rare hit loops.
template <typename T>
__global__ __launch_bounds__(kBlock) void zero_empty_fibres_kernel(int nfib, int K,
                                                                   const int32_t* __restrict__ pos2,
                                                                   T* __restrict__ out) {
  const int f = blockIdx.x * kBlock + threadIdx.x;
  if (f >= nfib || pos2[f + 1] > pos2[f]) return;
  for (int k = 0; k < K; ++k) out[(int64_t)f * K + k] = T(0);
}

// Ct[l * K + k] = C[k * L + l]
template <typename T>
__global__ __launch_bounds__(kBlock) void transpose_kernel(int K, int64_t L, const T* __restrict__ C,
                                                           T* __restrict__ Ct) {
  const int64_t idx = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (idx >= L * K) return;
  const int64_t l = idx / K;
  const int k = (int)(idx % K);
  Ct[idx] = C[(int64_t)k * L + l];
}

size_t ttm_workspace(Format f, const spt_tensor* B, int32_t K) {
  if (K < 1) K = 1;
  const int64_t nnz = B->nvals, L = B->level[2].N;
  size_t n = align_up((size_t)nnz * 4, 256) + align_up((size_t)L * K * 8, 256) +
             mttkrp_workspace(Format::COO2, B, K);
  if (f == Format::COO3) n += ttv_coo_workspace(nnz);
  return n + 256;
}

template <typename T>
static spt_status ttm_typed(Format f, const spt_tensor* B, const T* C, int K, int32_t* out_i,
                            int32_t* out_j, T* out_v, int64_t* out_nfib, void* ws, size_t ws_bytes,
                            hipStream_t s) {
  const int64_t nnz64 = B->nvals, L = B->level[2].N;
  if (nnz64 + kTtvChunk >= INT32_MAX) return fail(SPT_ERR_UNSUPPORTED, "ttm: more than 2^31 entries");
  const int nnz = (int)nnz64;
  if (nnz == 0) {
    if (out_nfib) {
      hipLaunchKernelGGL(set_i64_kernel, dim3(1), dim3(kWave), 0, s, out_nfib, (int64_t)0);
      SPT_CHECK_LAUNCH("ttm set count");
    }
    return SPT_OK;
  }
  if (!ws || ws_bytes < ttm_workspace(f, B, K))
    return fail(SPT_ERR_WORKSPACE, "ttm: workspace of %zu bytes needed, %zu given",
                ttm_workspace(f, B, K), ws_bytes);
  Workspace W(ws, ws_bytes);
  int32_t* fid = W.take<int32_t>(nnz);
  T* Ct = W.take<T>((size_t)L * K);
  if (f == Format::COO3) {
    const int nch = (nnz + kTtvChunk - 1) / kTtvChunk;
    int32_t* heads = W.take<int32_t>(nch);
    int32_t* off = W.take<int32_t>(nch);
    int32_t* scan_tmp = reinterpret_cast<int32_t*>(W.take<char>(scan_workspace(nch)));
    const int32_t *ci = B->level[0].crd, *cj = B->level[1].crd;
    const bool vec = ((reinterpret_cast<uintptr_t>(ci) | reinterpret_cast<uintptr_t>(cj)) & 15) == 0;
    if (vec) hipLaunchKernelGGL(ttv_count_kernel<true>, dim3(nch), dim3(kBlock), 0, s, nnz, ci, cj, heads);
    else hipLaunchKernelGGL(ttv_count_kernel<false>, dim3(nch), dim3(kBlock), 0, s, nnz, ci, cj, heads);
    SPT_CHECK_LAUNCH("ttm count");
    spt_status st = device_scan_i32<false>(heads, off, nch, scan_tmp, s);
    if (st != SPT_OK) return st;
    hipLaunchKernelGGL(ttv_total_kernel, dim3(1), dim3(kWave), 0, s, nch, heads, off, out_nfib);
    SPT_CHECK_LAUNCH("ttm total");
    if (vec)  // fid comes from the 256-byte aligned workspace
      hipLaunchKernelGGL(fiber_ids_kernel<true>, dim3(nch), dim3(kBlock), 0, s, nnz, ci, cj, off, fid,
                         out_i, out_j);
    else
      hipLaunchKernelGGL(fiber_ids_kernel<false>, dim3(nch), dim3(kBlock), 0, s, nnz, ci, cj, off, fid,
                         out_i, out_j);
    SPT_CHECK_LAUNCH("ttm fiber ids");
  } else {
    const int64_t nfib = B->level[2].M;
    if (nfib + 1 >= INT32_MAX) return fail(SPT_ERR_UNSUPPORTED, "ttm: tensor too large");
    if (out_nfib) {
      hipLaunchKernelGGL(set_i64_kernel, dim3(1), dim3(kWave), 0, s, out_nfib, nfib);
      SPT_CHECK_LAUNCH("ttm set count");
    }
    hipLaunchKernelGGL(expand_fiber_ids_kernel, dim3((unsigned)((nfib + kBlock - 1) / kBlock)),
                       dim3(kBlock), 0, s, (int)nfib, B->level[2].pos, fid);
    SPT_CHECK_LAUNCH("ttm expand fibre ids");
    hipLaunchKernelGGL(zero_empty_fibres_kernel<T>, dim3((unsigned)((nfib + kBlock - 1) / kBlock)),
                       dim3(kBlock), 0, s, (int)nfib, K, B->level[2].pos, out_v);
    SPT_CHECK_LAUNCH("ttm zero empty fibres");
  }
  hipLaunchKernelGGL(transpose_kernel<T>, dim3((unsigned)((L * K + kBlock - 1) / kBlock)),
                     dim3(kBlock), 0, s, K, L, C, Ct);
  SPT_CHECK_LAUNCH("ttm transpose");
  void* rest = static_cast<char*>(ws) + W.used;
  return mttkrp_typed<T>(Format::COO2, B, Ct, nullptr, K, out_v, rest, ws_bytes - W.used, s, fid,
                         B->level[2].crd);
}

spt_status ttm_dispatch(Format f, const spt_tensor* B, const void* C, int32_t K, int32_t* out_crd0,
                        int32_t* out_crd1, void* out_vals, int64_t* out_nfib_dev, void* ws,
                        size_t ws_bytes, hipStream_t s) {
  for (int k = 0; k < 3; ++k)
    if (!(B->level[k].flags & SPT_ORDERED))
      return fail(SPT_ERR_UNSUPPORTED, "ttm: every level of B must be ordered");
  if (B->dtype == SPT_F64)
    return ttm_typed<double>(f, B, static_cast<const double*>(C), K, out_crd0, out_crd1,
                             static_cast<double*>(out_vals), out_nfib_dev, ws, ws_bytes, s);
  return ttm_typed<float>(f, B, static_cast<const float*>(C), K, out_crd0, out_crd1,
                          static_cast<float*>(out_vals), out_nfib_dev, ws, ws_bytes, s);
}

// c held in LDS, one resident workgroup per compute unit (ttv_wave.hip)
bool ttv_wave_applies(int64_t nnz, int64_t K, int dtype);
size_t ttv_coo_wave_workspace(int64_t nnz);
size_t ttv_csf_wave_workspace(int64_t nnz);
template <typename T>
spt_status ttv_coo_wave(int64_t nnz, int64_t K, const int32_t* ci, const int32_t* cj, const int32_t* ck,
                        const T* vals, const T* c, int32_t* out_i, int32_t* out_j, T* out_v, int64_t* out_nnz,
                        void* ws, size_t ws_bytes, hipStream_t s);
template <typename T>
spt_status ttv_csf_wave(int64_t nnz, int64_t nfib, int64_t K, const int32_t* pos, const int32_t* ck,
                        const T* vals, const T* c, T* out_v, int64_t* out_count, void* ws, size_t ws_bytes,
                        hipStream_t s);

size_t ttv_workspace(Format f, const spt_tensor* B) {
  if (ttv_wave_applies(B->nvals, B->level[2].N, B->dtype))
    return f == Format::COO3 ? ttv_coo_wave_workspace(B->nvals) : ttv_csf_wave_workspace(B->nvals);
  return f == Format::COO3 ? ttv_coo_workspace(B->nvals) : seg_spmv_workspace(B->nvals);
}

spt_status ttv_dispatch(Format f, const spt_tensor* B, const void* c, int32_t* out_crd0,
                        int32_t* out_crd1, void* out_vals, int64_t* out_nnz_dev, void* ws,
                        size_t ws_bytes, hipStream_t s) {
  for (int k = 0; k < 3; ++k)
    if (!(B->level[k].flags & SPT_ORDERED))
      return fail(SPT_ERR_UNSUPPORTED, "ttv: every level of B must be ordered");
  if (f == Format::CSF3) {
    // The bottom level is a compressed level over the fibers: the same row
    // reduction as CSR SpMV with rows = fibers and x = c.
    const int64_t nfib = B->level[2].M;
    if (ttv_wave_applies(B->nvals, B->level[2].N, B->dtype)) {  // writes the count itself
      if (B->dtype == SPT_F64)
        return ttv_csf_wave<double>(B->nvals, nfib, B->level[2].N, B->level[2].pos, B->level[2].crd,
                                    static_cast<const double*>(B->vals), static_cast<const double*>(c),
                                    static_cast<double*>(out_vals), out_nnz_dev, ws, ws_bytes, s);
      return ttv_csf_wave<float>(B->nvals, nfib, B->level[2].N, B->level[2].pos, B->level[2].crd,
                                 static_cast<const float*>(B->vals), static_cast<const float*>(c),
                                 static_cast<float*>(out_vals), out_nnz_dev, ws, ws_bytes, s);
    }
    if (out_nnz_dev) {
      hipLaunchKernelGGL(set_i64_kernel, dim3(1), dim3(kWave), 0, s, out_nnz_dev, nfib);
      SPT_CHECK_LAUNCH("ttv set count");
    }
    return csr_rows_reduce(B->dtype, B->nvals, nfib, B->level[2].pos, B->level[2].crd, B->vals, c,
                           out_vals, ws, ws_bytes, s);
  }
  if (ttv_wave_applies(B->nvals, B->level[2].N, B->dtype)) {
    const int32_t *ci = B->level[0].crd, *cj = B->level[1].crd, *ck = B->level[2].crd;
    if (B->dtype == SPT_F64)
      return ttv_coo_wave<double>(B->nvals, B->level[2].N, ci, cj, ck, static_cast<const double*>(B->vals),
                                  static_cast<const double*>(c), out_crd0, out_crd1,
                                  static_cast<double*>(out_vals), out_nnz_dev, ws, ws_bytes, s);
    return ttv_coo_wave<float>(B->nvals, B->level[2].N, ci, cj, ck, static_cast<const float*>(B->vals),
                               static_cast<const float*>(c), out_crd0, out_crd1, static_cast<float*>(out_vals),
                               out_nnz_dev, ws, ws_bytes, s);
  }
  if (B->dtype == SPT_F64)
    return ttv_coo_typed<double>(B, static_cast<const double*>(c), out_crd0, out_crd1,
                                 static_cast<double*>(out_vals), out_nnz_dev, ws, ws_bytes, s);
  return ttv_coo_typed<float>(B, static_cast<const float*>(c), out_crd0, out_crd1,
                              static_cast<float*>(out_vals), out_nnz_dev, ws, ws_bytes, s);
}

}  // namespace spt
