// Dense best-matching-unit search, fp32 pass, fast variant for dim % 4 == 0 and 16-byte aligned
// operands (paper: BMU equation; "Parallelism": distances through linear algebra).
//
// Same computation, modes, tiling and outputs as k_bmu_dense in bmu_dense.hip; what differs is
// how the operand tiles reach LDS.  gfx950 can load 16 bytes per lane from global memory
// straight into LDS (global_load_lds_dwordx4): no staging registers, no LDS store instructions,
// and the latency of the loads is decoupled from the instruction stream - a wavefront only
// waits for its own loads right before the workgroup barrier that publishes the buffer.
//
// Such a load writes lane l's 16 bytes to LDS base + 16 l, so one instruction fills 1 KB =
// eight tile rows of kBK = 32 floats, without room for padding.  Bank conflicts of the
// ds_read_b128 operand reads (32 lanes read the same column chunk of 32 different rows) are
// avoided by a swizzle instead: the 16-byte chunk q of row r is stored at chunk position
// q ^ swz(r), swz(r) = (r & 7) ^ ((r >> 3) & 1).  The loading lane simply picks the global
// chunk that belongs at its LDS position.  Rows and columns outside the matrices are read from
// a 16-byte block of zeros.
#include "bmu_dense_common.hpp"

namespace som {

typedef __attribute__((address_space(3))) void *lptr_t;

constexpr int kTileFloats = kTN * kBK;        // one operand tile in LDS: 128 rows x 32 floats = 16 KB
static_assert(kTN == kTI, "both operand tiles have the same shape");

__device__ __forceinline__ unsigned lds_address(const float *p) { return (unsigned)(size_t)(lptr_t)p; }

// One direct-to-LDS load: lane l's 16 bytes at `g` go to LDS byte address lds_base + 16 l
// (lds_base wavefront-uniform, passed in M0).  Written as inline assembly on purpose: the
// compiler would otherwise make every later LDS read wait for these loads, although they fill
// the buffer that is NOT being read; the ordering that matters is enforced by hand
// (wait_vector_memory() before the barrier that publishes the buffer).  M0 is a reserved
// register that the compiler reloads before each use of its own, so overwriting it is safe.
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void load16_to_lds(const float *g, unsigned lds_base) {
  asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(g), "s"(lds_base) : "memory", "m0");
}
#pragma clang diagnostic pop

__device__ __forceinline__ void wait_vector_memory() {
  // s_waitcnt vmcnt(0): every vector memory operation of this wavefront, the direct-to-LDS
  // loads included, has completed (expcnt and lgkmcnt fields left at their maxima)
  __builtin_amdgcn_s_waitcnt(0x0F70);
}

template <bool kCollect>
__global__ __launch_bounds__(256, 2) void k_bmu_dense_dl(const float *__restrict__ X, const float *__restrict__ Wc,
                                                         const float *__restrict__ wc,
                                                         const float *__restrict__ zero16, int64_t n, int k,
                                                         int dim, CandView out, const int32_t *__restrict__ rows,
                                                         const int32_t *__restrict__ n_slots,
                                                         const float *__restrict__ thr, int32_t *__restrict__ cnt,
                                                         int32_t *__restrict__ list, float *__restrict__ dump) {
  __shared__ __attribute__((aligned(16))) float sW[2][kTileFloats];
  __shared__ __attribute__((aligned(16))) float sX[2][kTileFloats];
  __shared__ float sWn[2][kTN];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1;          // which 64-node half of the tile
  const int wi = wave & 1;           // which 64-instance half of the tile
  const int l32 = lane & 31;
  const int lhi = lane >> 5;
  const int64_t inst0 = (int64_t)blockIdx.x * kTI;
  const int64_t n_inst = kCollect ? (int64_t)*n_slots : n;
  if (inst0 >= n_inst) return;       // uniform over the workgroup

  const int nK = (dim + kBK - 1) / kBK;
  const int nNB_all = (k + kTN - 1) / kTN;
  const int nb_per = (nNB_all + (int)gridDim.y - 1) / (int)gridDim.y;
  const int nb_first = (int)blockIdx.y * nb_per;
  const int nNB = min(nb_per, nNB_all - nb_first);
  if (nNB <= 0) return;              // uniform over the workgroup
  const int total = nK * nNB;

  // ---- loader: wavefront w issues instructions i = 0..3 per operand; instruction (w, i) fills
  // rows 8 (4 w + i) .. + 7 of the tile; lane l sits at row + (l >> 3), chunk position l & 7.
  const int ld_rloc = lane >> 3;
  const int ld_pos = lane & 7;
  const float *xp[4];
  const float *wp[4];
  bool xok[4], wok[4];
  int wrow[4];       // tile-local row of this lane for instruction i
  int ld_col[4];     // first column (within a chunk of 32) this lane fetches for instruction i
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int row = 8 * (4 * wave + i) + ld_rloc;
    wrow[i] = row;
    ld_col[i] = 4 * (ld_pos ^ ((row & 7) ^ ((row >> 3) & 1)));
    const int64_t slot = inst0 + row;
    xok[i] = slot < n_inst;
    const int64_t xr = kCollect ? (xok[i] ? (int64_t)rows[slot] : 0) : (xok[i] ? slot : 0);
    xp[i] = X + xr * dim;
    wok[i] = false;
    wp[i] = Wc;
  }
  const unsigned lds_w = lds_address(&sW[0][1024 * wave]);    // this wavefront's 4 KB slice of buffer 0
  const unsigned lds_x = lds_address(&sX[0][1024 * wave]);
  int ld_nb = nb_first, ld_kc = 0;                              // position of the next chunk to load
  auto issue_loads = [&](int buf) {
    if (ld_kc == 0) {                                           // entering a node block
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int64_t node = (int64_t)ld_nb * kTN + wrow[i];
        wok[i] = node < k;
        wp[i] = Wc + (wok[i] ? node : 0) * dim;
      }
      if (tid < kTN) {
        const int node = ld_nb * kTN + tid;
        sWn[ld_nb & 1][tid] = node < k ? wc[node] : INFINITY;    // padded nodes can never win
      }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int c = ld_kc * kBK + ld_col[i];
      const bool cok = c < dim;
      load16_to_lds((wok[i] && cok) ? wp[i] + c : zero16, lds_w + buf * (kTileFloats * 4) + i * 1024);
      load16_to_lds((xok[i] && cok) ? xp[i] + c : zero16, lds_x + buf * (kTileFloats * 4) + i * 1024);
    }
    if (++ld_kc == nK) { ld_kc = 0; ++ld_nb; }
  };

  // ---- reader: lane (l32, lhi) needs columns 8 g + 4 lhi .. + 3 of rows l32 (+32) of its halves
  const int rd_swz = (l32 & 7) ^ ((l32 >> 3) & 1);
  int rd_off[4];
#pragma unroll
  for (int g = 0; g < 4; ++g) rd_off[g] = 4 * ((2 * g + lhi) ^ rd_swz);
  const int a_base = (wm * 64 + l32) * kBK;
  const int b_base = (wi * 64 + l32) * kBK;

  const float kMinusTwo[2] = {-2.f, -2.f};
  Top2 top[2];
  float lim[2];
  int64_t slot_of[2];
#pragma unroll
  for (int ni = 0; ni < 2; ++ni) {
    top2_init(top[ni]);
    slot_of[ni] = inst0 + wi * 64 + ni * 32 + l32;
    lim[ni] = (kCollect && slot_of[ni] < n_inst) ? thr[slot_of[ni]] : -INFINITY;
  }

  f32x16 acc[2][2], tot[2][2];
#pragma unroll
  for (int mi = 0; mi < 2; ++mi)
#pragma unroll
    for (int ni = 0; ni < 2; ++ni)
#pragma unroll
      for (int v = 0; v < 16; ++v) { acc[mi][ni][v] = 0.f; tot[mi][ni][v] = 0.f; }

  issue_loads(0);
  wait_vector_memory();
  __syncthreads();

  for (int t = 0; t < total; ++t) {
    const int nb = nb_first + t / nK, kc = t % nK;
    if (t + 1 < total) issue_loads((t + 1) & 1);

    const float *pw = &sW[t & 1][a_base];
    const float *px = &sX[t & 1][b_base];
    f32x4 a[2][2], b[2][2];          // [register set][32-row block]
    a[0][0] = *reinterpret_cast<const f32x4 *>(pw + rd_off[0]);
    a[0][1] = *reinterpret_cast<const f32x4 *>(pw + 32 * kBK + rd_off[0]);
    b[0][0] = *reinterpret_cast<const f32x4 *>(px + rd_off[0]);
    b[0][1] = *reinterpret_cast<const f32x4 *>(px + 32 * kBK + rd_off[0]);
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int cur = g & 1, nxt = cur ^ 1;
      if (g < 3) {                   // operands of the next group arrive while this group multiplies
        a[nxt][0] = *reinterpret_cast<const f32x4 *>(pw + rd_off[g + 1]);
        a[nxt][1] = *reinterpret_cast<const f32x4 *>(pw + 32 * kBK + rd_off[g + 1]);
        b[nxt][0] = *reinterpret_cast<const f32x4 *>(px + rd_off[g + 1]);
        b[nxt][1] = *reinterpret_cast<const f32x4 *>(px + 32 * kBK + rd_off[g + 1]);
      }
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[cur][0][s], b[cur][0][s], acc[0][0], 0, 0, 0);
        acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[cur][0][s], b[cur][1][s], acc[0][1], 0, 0, 0);
        acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[cur][1][s], b[cur][0][s], acc[1][0], 0, 0, 0);
        acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[cur][1][s], b[cur][1][s], acc[1][1], 0, 0, 0);
      }
    }

    const bool last_k = (kc == nK - 1);
    if (last_k || (kc % kFlushChunks) == kFlushChunks - 1) {
#pragma unroll
      for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
#pragma unroll
          for (int v = 0; v < 16; ++v) { tot[mi][ni][v] += acc[mi][ni][v]; acc[mi][ni][v] = 0.f; }
    }
    if (last_k) consume_scores<kCollect>(tot, sWn[nb & 1], nb * kTN, k, wm, lhi, kMinusTwo, top, lim, slot_of, cnt, list, dump, n);

    wait_vector_memory();
    __syncthreads();
  }
  if (kCollect) return;
  merge_and_store<kTI>(top, &sW[0][0], reinterpret_cast<int *>(&sX[0][0]), tid, wm, wi, l32, lhi, inst0, n, blockIdx.y,
                  out);
}

hipError_t launch_bmu_dense_dl(som_ctx *c, const float *X, int64_t n, dim3 grid, bool collect, float *dump) {
  if (collect) {
    CandView out{nullptr, nullptr, nullptr};
    hipLaunchKernelGGL((k_bmu_dense_dl<true>), grid, dim3(256), 0, c->stream, X, c->Wc, c->wn32, c->zero16, n, c->k,
                       c->dim, out, c->collect_rows, c->list_counts + 1, c->collect_thr, c->collect_cnt,
                       c->collect_list, nullptr);
  } else {
    CandView out{c->cand_val, c->cand_idx, c->cand_over};
    hipLaunchKernelGGL((k_bmu_dense_dl<false>), grid, dim3(256), 0, c->stream, X, c->Wc, c->wn32, c->zero16, n, c->k,
                       c->dim, out, nullptr, nullptr, nullptr, nullptr, nullptr, dump);
  }
  return hipGetLastError();
}

}  // namespace som
