// C = A * B^T as in k_gemm for deep reductions (K >= 1024), with the operand tiles brought from global
// memory straight into LDS (global_load_lds_dwordx4: lane l's 16 bytes land at the wave's LDS base
// + 16*l, no registers in between) through a ring of NST stages, so that NST-1 k-steps of 64 are in
// flight per block.
//
// Stage layout: A region [BM rows][8 chunks of 8 elements], B region [BN rows][8 chunks], rows 128
// bytes apart with no padding.  One wave instruction fills 8 rows (lane = row*8 + position); the
// lane at (row, position) fetches the row's chunk  position ^ ((row >> 1) & 7), so that the MFMA
// operand reads (32 consecutive rows, one chunk) touch every LDS bank exactly once.  Rows beyond
// the matrix, taps in the padding and k >= K are fetched from a page of zeros.
//
// The compiler orders every LDS access of a wave after all of that wave's outstanding LDS-writing
// loads, which would drain the ring at each step if one wave did both; here the loads belong to
// loader waves, whose only waits are explicit (s_waitcnt vmcnt(loads of the younger stages)).
#pragma once
#include "gemm.hip.h"

// cache-policy operand of an LDS-writing load: non-temporal, for data that is read once per launch
#define LOAD_NT 2
#define GLOBAL_AS(p) ((const void __attribute__((address_space(1)))*)(p))
#define LDS_AS(p) ((void __attribute__((address_space(3)))*)(p))

// wait until at most N of this wave's vector-memory loads are outstanding (expcnt, lgkmcnt untouched)
template <int N>
__device__ __forceinline__ void vm_wait() {
  static_assert(N >= 0 && N < 64, "vmcnt range");
  __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

// wait until at most n (wave-uniform, < 64) of this wave's vector-memory operations are outstanding
__device__ __forceinline__ void vm_wait_dyn(int n) {
  switch (n) {
#define VMW(i) case i: vm_wait<i>(); break;
#define VMW8(b) VMW(b) VMW(b + 1) VMW(b + 2) VMW(b + 3) VMW(b + 4) VMW(b + 5) VMW(b + 6) VMW(b + 7)
    VMW8(0) VMW8(8) VMW8(16) VMW8(24) VMW8(32) VMW8(40) VMW8(48) VMW8(56)
#undef VMW8
#undef VMW
    default: vm_wait<0>(); break;
  }
}

// The two jobs of a block belong to different waves: WGM x WGN compute waves (MFMAs on operands read
// from the ring with ordinary LDS reads, all reads of a k-step before its first MFMA) and four loader
// waves that do nothing but keep NST-1 stages of LDS-writing loads in flight.  A wave that did both
// would spend some hundred cycles per stage issuing its loads, computing nothing meanwhile.  One
// barrier per k-step: the loaders arrive when their part of stage kt has landed, the compute waves
// when they are done with stage kt-1 (whose slot the loaders refill next).
template <int BM, int BN, int WGM, int WGN, int NST, class AL, class EP>
__global__ __launch_bounds__((WGM * WGN + 4) * 64) void k_gemm_rs(AL al, const bf16_t* __restrict__ Bm_, int64_t ldb_, int N, EP ep,
                                                                  const bf16_t* __restrict__ zpage) {
  constexpr int NCW = WGM * WGN, NLW = 4, THREADS = (NCW + NLW) * 64;
  constexpr int TM = BM / (WGM * 32), TN = BN / (WGN * 32);
  static_assert((NCW == 4 || NCW == 8) && TM >= 1 && TN >= 1 && NST >= 2 && NST <= 8, "tile shape");
  constexpr int BK = 64;
  constexpr int AI = BM / 32, BI = BN / 32;  // loads per loader wave per stage (8 rows each)
  constexpr int A_BYTES = BM * 128, B_BYTES = BN * 128, ST_BYTES = A_BYTES + B_BYTES;
  constexpr int D = NST - 1;                 // stages in flight
  static_assert(BM * (BN + 8) * 2 <= NST * ST_BYTES, "staging tile must fit in the ring");
  static_assert(D * (AI + BI) < 64, "vmcnt range");
  static_assert(AI % 2 == 0, "row groups per wave");
  extern __shared__ __attribute__((aligned(16))) bf16_t ring[];
  __shared__ int64_t rowoff[BM];
  __shared__ int rowcols[BM];

  const typename AL::Cls acls = al.cls(blockIdx.z);
  const auto mcls = ep.map.cls(blockIdx.z);
  const int m0 = blockIdx.x * BM, n0 = blockIdx.y * BN;
  if (m0 >= acls.M) return;
  const int K = acls.K, nk = (K + BK - 1) / BK;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  char* const ring_b = reinterpret_cast<char*>(ring);
  const bool compute = wave < NCW;
  const int wm = compute ? wave / WGN : 0, wn = compute ? wave % WGN : 0;
  f32x16_t acc[TM][TN];

  if (!compute) {
    // ------------------------------------------------------------------ loaders
    const int lw = wave - NCW;
    const bf16_t* Bm = al.bmat(acls, Bm_);
    const int64_t ldb = (Bm == Bm_) ? ldb_ : (int64_t)K;
    const int dr = lane >> 3, dpos = lane & 7;
    // rows r = (lw*AI + j)*8 + dr: the permutation (r >> 1) & 7 depends on j only through its parity
    typename AL::Row arow[AI];
#pragma unroll
    for (int j = 0; j < AI; ++j) arow[j] = al.row(m0 + (lw * AI + j) * 8 + dr, acls);
    typename AL::KCur acur[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) acur[j] = al.kcur((dpos ^ ((j * 4 + (dr >> 1)) & 7)) * 8, acls);
    const bf16_t* brow[BI];
    int b_k[BI];
#pragma unroll
    for (int j = 0; j < BI; ++j) {
      const int r = (lw * BI + j) * 8 + dr, n = n0 + r;
      brow[j] = (n < N) ? Bm + (int64_t)n * ldb : nullptr;
      b_k[j] = (dpos ^ ((r >> 1) & 7)) * 8;
    }
    // stages are issued in order of k, so the column cursors simply step along
    auto issue = [&](int stage, int k0) __attribute__((always_inline)) {
      char* sb = ring_b + stage * ST_BYTES;
#pragma unroll
      for (int j = 0; j < AI; ++j) {
        const bf16_t* p = al.addr(arow[j], acur[j & 1], acls);
        if (!p) p = zpage;
        __builtin_amdgcn_global_load_lds(GLOBAL_AS(p), LDS_AS(sb + (lw * AI + j) * 1024), 16, 0, 0);
      }
#pragma unroll
      for (int j = 0; j < BI; ++j) {
        const int k = k0 + b_k[j];
        const bf16_t* p = (brow[j] && k < K) ? brow[j] + k : zpage;
        __builtin_amdgcn_global_load_lds(GLOBAL_AS(p), LDS_AS(sb + A_BYTES + (lw * BI + j) * 1024), 16, 0, 0);
      }
      al.kstep(acur[0], BK, acls);
      al.kstep(acur[1], BK, acls);
    };
    int st_next = 0;  // slot of the next stage to issue
    for (int s = 0; s < D && s < nk; ++s) { issue(st_next, s * BK); st_next = st_next == NST - 1 ? 0 : st_next + 1; }
    for (int kt = 0; kt < nk; ++kt) {
      const int younger = min(D - 1, nk - 1 - kt);  // stages issued after stage kt
      vm_wait_dyn(younger * (AI + BI));
      __builtin_amdgcn_s_barrier();  // stage kt has landed; the compute waves have left stage kt - 1
      if (kt + D < nk) { issue(st_next, (kt + D) * BK); st_next = st_next == NST - 1 ? 0 : st_next + 1; }
    }
  } else {
    // ------------------------------------------------------------------ compute waves
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
    f32x16_t acc2;
#pragma unroll
    for (int e = 0; e < 16; ++e) acc2[e] = 0.f;
    // operand read offsets within a stage: row (tile*32 + lane%32), chunk (ks*2 + lane/32) ^ permutation
    const int l32 = lane & 31, h = lane >> 5, sw = (l32 >> 1) & 7;
    int rd[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) rd[ks] = l32 * 128 + (((ks * 2 + h) ^ sw) * 16);
    const int offA = wm * TM * 4096, offB = A_BYTES + wn * TN * 4096;
    int st = 0;
    for (int kt = 0; kt < nk; ++kt) {
      __builtin_amdgcn_s_barrier();  // stage kt is in LDS
      const char* sA = ring_b + st * ST_BYTES + offA;
      const char* sB = ring_b + st * ST_BYTES + offB;
      // all operand reads of the stage first (one LDS latency per k-step, not one per MFMA)
      bf16x8_t a[4][TM], b[4][TN];
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
#pragma unroll
        for (int i = 0; i < TM; ++i) a[ks][i] = *reinterpret_cast<const bf16x8_t*>(sA + rd[ks] + i * 4096);
#pragma unroll
        for (int j = 0; j < TN; ++j) b[ks][j] = *reinterpret_cast<const bf16x8_t*>(sB + rd[ks] + j * 4096);
      }
#pragma unroll
      for (int ks = 0; ks < 4; ++ks)
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j) {
            // a lone tile alternates between two accumulators: consecutive MFMAs do not wait for each other
            if (TM * TN == 1 && (ks & 1)) acc2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[ks][j], a[ks][i], acc2, 0, 0, 0);
            else acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[ks][j], a[ks][i], acc[i][j], 0, 0, 0);
          }
      st = (st == NST - 1) ? 0 : st + 1;
    }
    if (TM * TN == 1) {
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[0][0][e] += acc2[e];
    }
  }
  __syncthreads();  // every wave is done with the ring, which becomes the staging tile
  gemm_epilogue<BM, BN, TM, TN, THREADS>(acc, ep, mcls, m0, n0, N, wm, wn, ring, rowoff, rowcols, compute);
}
