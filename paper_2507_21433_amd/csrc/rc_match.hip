// rc_match_blocks: query-block x pool-block score contraction on the matrix cores with a fused
// top-1 / runner-up / threshold selection (ReasonCache Sec. IV-A Stage 2: with the squared norms
// cached, comparing two blocks only needs the dot product of the flattened tensors).
//
// Shape of the work per layer: S[P x Q] = Xp[P x D] * Xq[Q x D]^T for the K tensors and again for
// the V tensors; both operands are contiguous along the reduction dimension.  Pool blocks are the
// rows of the MFMA tile (they land in the accumulator registers of a lane), query blocks are the
// columns (they land on lanes), so the argmax over the pool is mostly an in-lane reduction.
//
// One workgroup owns a BP x BQ tile of S for the whole reduction (no split-K, so the selection
// can be fused).  Operand slices of 64 elements (128 bytes per block) are copied global -> LDS
// with direct-to-LDS 16-byte loads into a two-stage ring; the 16-byte chunks of a row are
// XOR-swizzled by the row number so that the 32 rows a fragment read touches hit distinct banks.
//
// K and V are normalised by different norms but share one accumulator tile: after the K
// phase the accumulators are multiplied by (aKq aKp)/(aVq aVp), the V phase continues into
// them, and the epilogue multiplies by aVq aVp / 2, with a = 1/sqrt(squared norm).
#include <hip/hip_runtime.h>

#include "rc_common.hpp"

namespace rc {
namespace {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

#define RC_GLOBAL_PTR(p) ((const __attribute__((address_space(1))) void*)(p))
#define RC_LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))

constexpr int kBK = 64;             // reduction elements per pipeline step
constexpr int kRowBytes = kBK * 2;  // bytes of one block's slice in LDS
constexpr int kSrdFlags = 0x00020000;  // raw 32-bit buffer descriptor word 3

// Partial selection result of one pool tile for one query.
struct Part {
  float best;
  int idx;
  float second;
  int pad;
};

struct MatchParams {
  const char *kq, *vq, *kp, *vp;
  const float *q_ksq, *q_vsq, *p_ksq, *p_vsq;
  const uint8_t* live;
  Part* part;                      // [L][npt][Q]
  long long q_lstride_b, p_lstride_b;  // bytes between layers
  int L, Q, P;
  int T, H;
  int npt, nqt;
  int total;  // L * npt * nqt
  int chunk;  // tiles handed to one XCD in a row
};

__device__ __forceinline__ void top2_push(float v, int i, float& best, int& bidx, float& second) {
  const bool gt = v > best;
  second = gt ? best : fmaxf(second, v);
  bidx = gt ? i : bidx;
  best = gt ? v : best;
}

// Merge (b2, i2, s2) into (best, bidx, second): higher score wins, equal scores go to the lower index.
__device__ __forceinline__ void top2_merge(float& best, int& bidx, float& second, float b2, int i2, float s2) {
  const bool take = (b2 > best) || (b2 == best && (unsigned)i2 < (unsigned)bidx);
  const float loser = take ? best : b2;
  const float wsec = take ? s2 : second;
  bidx = take ? i2 : bidx;
  best = take ? b2 : best;
  second = fmaxf(wsec, loser);
}

template <bool BF16>
__device__ __forceinline__ f32x16 mfma(uint4 a, uint4 b, f32x16 c) {
  if (BF16)
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
  else
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}

__device__ __forceinline__ float inv_sqrt_or(float sq, float if_zero) { return sq > 0.f ? 1.0f / sqrtf(sq) : if_zero; }

}  // namespace

// BP x BQ tile, WP x WQ waves, each wave (BP/WP) x (BQ/WQ).  MODE 0 = block score, 1 = per-head-all.
template <bool BF16, int BP, int BQ, int WP, int WQ, int MODE, int MINBLK>
__global__ __launch_bounds__(64 * WP * WQ, MINBLK) void match_tile_kernel(const MatchParams p) {
#if defined(__HIP_DEVICE_COMPILE__)  // the host pass only needs the launch stub (buffer-resource types are device-only)
  constexpr int NT = 64 * WP * WQ;
  constexpr int WTP = BP / WP, WTQ = BQ / WQ;
  constexpr int TP = WTP / 32, TQ = WTQ / 32;
  constexpr int LA = BP * 8 / NT, LB = BQ * 8 / NT;  // 16-byte loads per thread per step
  static_assert(BP % (32 * WP) == 0 && BQ % (32 * WQ) == 0, "wave tiles are multiples of 32");
  static_assert((BP * 8) % NT == 0 && (BQ * 8) % NT == 0, "loads divide evenly");
  static_assert(NT >= BQ, "one thread per query column in the tile epilogue");

  // Separate arrays per stage so that reads of one stage are known not to alias the
  // direct-to-LDS writes into the other.
  __shared__ __attribute__((aligned(1024))) char sA0[BP * kRowBytes];
  __shared__ __attribute__((aligned(1024))) char sB0[BQ * kRowBytes];
  __shared__ __attribute__((aligned(1024))) char sA1[BP * kRowBytes];
  __shared__ __attribute__((aligned(1024))) char sB1[BQ * kRowBytes];
  __shared__ float s_rp[BP], s_fp[BP], s_bias[BP];  // pool rows: K/V ratio, final scale, -inf for dead/tail
  __shared__ float s_rq[BQ], s_fq[BQ];              // query columns
  __shared__ Part s_part[WP][BQ];

  // ---- which tile: consecutive runs of `chunk` tiles go to one XCD (workgroups are dealt
  // round-robin to the 8 XCDs), so tiles that share operands share an L2.
  const int wg = blockIdx.x;
  const int slot = wg >> 3;
  const int tile = ((slot / p.chunk) * 8 + (wg & 7)) * p.chunk + slot % p.chunk;
  if (tile >= p.total) return;
  const int qt = tile % p.nqt;
  const int pt = (tile / p.nqt) % p.npt;
  const int l = tile / (p.nqt * p.npt);
  const int p0 = pt * BP, q0 = qt * BQ;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wp = wave / WQ, wq = wave % WQ;

  const int D = p.T * p.H * 128;
  const long long row_b = (long long)D * 2;
  const int rowsA = min(BP, p.P - p0), rowsB = min(BQ, p.Q - q0);

  // ---- buffer resources over this tile's rows of the four tensors (index 0 = K, 1 = V).  The
  // range check of the buffer unit is a second guard; offsets are kept inside the rows anyway.
  const long long offPool = l * p.p_lstride_b + (long long)p0 * row_b;
  const long long offQry = l * p.q_lstride_b + (long long)q0 * row_b;
  __amdgpu_buffer_rsrc_t resA[2], resB[2];
  resA[0] = __builtin_amdgcn_make_buffer_rsrc((void*)(p.kp + offPool), 0, (int)(rowsA * row_b), kSrdFlags);
  resA[1] = __builtin_amdgcn_make_buffer_rsrc((void*)(p.vp + offPool), 0, (int)(rowsA * row_b), kSrdFlags);
  resB[0] = __builtin_amdgcn_make_buffer_rsrc((void*)(p.kq + offQry), 0, (int)(rowsB * row_b), kSrdFlags);
  resB[1] = __builtin_amdgcn_make_buffer_rsrc((void*)(p.vq + offQry), 0, (int)(rowsB * row_b), kSrdFlags);

  // ---- per-thread source offsets of the direct-to-LDS loads.  Load i of a wave fills LDS rows
  // (i*NT + wave*64)/8 .. +7, lane -> (row lane/8, physical chunk lane%8); the logical chunk
  // fetched is physical ^ (row & 7).  Rows past the end of the pool / queries re-read the last
  // valid row (their results are masked), so no load leaves the tensors.
  const uint32_t swz = (uint32_t)(((lane & 7) ^ (lane >> 3)) * 16);
  uint32_t offA[LA], offB[LB];
#pragma unroll
  for (int i = 0; i < LA; ++i) offA[i] = (uint32_t)min((i * NT + tid) >> 3, rowsA - 1) * (uint32_t)row_b + swz;
#pragma unroll
  for (int i = 0; i < LB; ++i) offB[i] = (uint32_t)min((i * NT + tid) >> 3, rowsB - 1) * (uint32_t)row_b + swz;

  // ---- fragment read offsets: lane -> row lane%32 of a 32-row group, 16-byte chunk (2*kk + lane/32)
  const uint32_t fragA = (uint32_t)((wp * WTP + (lane & 31)) * kRowBytes);
  const uint32_t fragB = (uint32_t)((wq * WTQ + (lane & 31)) * kRowBytes);
  // ---- steps.  A phase is one tensor (K or V) of the whole block (MODE 0) or of one head
  // (MODE 1).  Step u of a phase reads 128 bytes per block at byte offset
  // base + (u/2)*tok + (u%2)*128:  tok = 256, base = 0 walks the flattened block; tok = H*256,
  // base = head*256 walks one head's [T][Dh] slice.
  const int sps = (MODE == 0) ? (D / kBK) : (p.T * 2);
  const int tok = (MODE == 0) ? 256 : p.H * 256;
  auto step_off = [&](int base, int u) { return base + (u >> 1) * tok + (u & 1) * 128; };

  auto issue = [&](const __amdgpu_buffer_rsrc_t ra, const __amdgpu_buffer_rsrc_t rb, int off, char* dA, char* dB) {
#pragma unroll
    for (int i = 0; i < LA; ++i)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(ra, RC_LDS_PTR(dA + (i * NT + wave * 64) * 16), 16, offA[i], off, 0, 0);
#pragma unroll
    for (int i = 0; i < LB; ++i)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rb, RC_LDS_PTR(dB + (i * NT + wave * 64) * 16), 16, offB[i], off, 0, 0);
  };

  f32x16 acc[TP][TQ];
#pragma unroll
  for (int i = 0; i < TP; ++i)
#pragma unroll
    for (int j = 0; j < TQ; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // Fragments of sub-step kk+1 are requested before the matrix instructions of sub-step kk are
  // issued; the scheduling barriers keep the compiler from hoisting every read to the top.
  auto load_frags = [&](const char* sA, const char* sB, int kk, uint4 (&af)[TP], uint4 (&bf)[TQ]) {
    const uint32_t c = (uint32_t)(((2 * kk + (lane >> 5)) ^ (lane & 7)) * 16);
#pragma unroll
    for (int i = 0; i < TP; ++i) af[i] = *reinterpret_cast<const uint4*>(sA + fragA + i * 32 * kRowBytes + c);
#pragma unroll
    for (int j = 0; j < TQ; ++j) bf[j] = *reinterpret_cast<const uint4*>(sB + fragB + j * 32 * kRowBytes + c);
  };
  auto compute = [&](const char* sA, const char* sB) {
    uint4 af[2][TP], bf[2][TQ];
    load_frags(sA, sB, 0, af[0], bf[0]);
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      if (kk + 1 < 4) load_frags(sA, sB, kk + 1, af[(kk + 1) & 1], bf[(kk + 1) & 1]);
#pragma unroll
      for (int i = 0; i < TP; ++i)
#pragma unroll
        for (int j = 0; j < TQ; ++j) acc[i][j] = mfma<BF16>(af[kk & 1][i], bf[kk & 1][j], acc[i][j]);
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  // ---- scale factors of the current head (or of the whole block) into LDS
  auto load_scales = [&](int head) {
    const int nh = (MODE == 0) ? 1 : p.H;
    for (int r = tid; r < BP; r += NT) {
      const int gp = p0 + r;
      float rp = 0.f, fp = 0.f, bias = -INFINITY;
      if (gp < p.P) {
        const long long o = ((long long)l * p.P + gp) * nh + head;
        const float ak = inv_sqrt_or(p.p_ksq[o], 0.f), av = inv_sqrt_or(p.p_vsq[o], 1.f);
        rp = ak / av;
        fp = av;
        if (!p.live || p.live[(long long)l * p.P + gp]) bias = 0.f;
      }
      s_rp[r] = rp;
      s_fp[r] = fp;
      s_bias[r] = bias;
    }
    for (int c = tid; c < BQ; c += NT) {
      const int gq = q0 + c;
      float rq = 0.f, fq = 0.f;
      if (gq < p.Q) {
        const long long o = ((long long)l * p.Q + gq) * nh + head;
        const float ak = inv_sqrt_or(p.q_ksq[o], 0.f), av = inv_sqrt_or(p.q_vsq[o], 1.f);
        rq = ak / av;
        fq = 0.5f * av;
      }
      s_rq[c] = rq;
      s_fq[c] = fq;
    }
  };

  // rows of accumulator register group g (4 registers) of row tile i: wp*WTP + i*32 + 8*g + 4*(lane/32) + 0..3
  auto row_of = [&](int i, int g) { return wp * WTP + i * 32 + 8 * g + 4 * (lane >> 5); };

  // the 16 pool-row factors of row tile i as one register tuple, matching an accumulator tile
  auto row_vec = [&](const float* tab, int i) {
    f32x16 v;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const f32x4 t = *reinterpret_cast<const f32x4*>(&tab[row_of(i, g)]);
#pragma unroll
      for (int e = 0; e < 4; ++e) v[4 * g + e] = t[e];
    }
    return v;
  };

  // acc <- acc * (rq * rp)   (end of a K phase)
  auto rescale = [&]() {
    float rq[TQ];
#pragma unroll
    for (int j = 0; j < TQ; ++j) rq[j] = s_rq[wq * WTQ + j * 32 + (lane & 31)];
#pragma unroll
    for (int i = 0; i < TP; ++i) {
      const f32x16 rp = row_vec(s_rp, i);
#pragma unroll
      for (int j = 0; j < TQ; ++j) {
        acc[i][j] = acc[i][j] * (rp * rq[j]);
        __builtin_amdgcn_sched_barrier(0);  // one tile at a time keeps the register pressure low
      }
    }
  };

  // per-head mode: running minimum over heads of the finished head score; acc restarts at 0
  f32x16 smin[MODE == 0 ? 1 : TP][MODE == 0 ? 1 : TQ];
  if (MODE == 1) {
#pragma unroll
    for (int i = 0; i < TP; ++i)
#pragma unroll
      for (int j = 0; j < TQ; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) smin[i][j][r] = INFINITY;
  }
  auto finish_head = [&]() {
    float fq[TQ];
#pragma unroll
    for (int j = 0; j < TQ; ++j) fq[j] = s_fq[wq * WTQ + j * 32 + (lane & 31)];
#pragma unroll
    for (int i = 0; i < TP; ++i)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const f32x4 fp = *reinterpret_cast<const f32x4*>(&s_fp[row_of(i, g)]);
#pragma unroll
        for (int j = 0; j < TQ; ++j)
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float s = acc[i][j][4 * g + e] * (fq[j] * fp[e]);
            smin[MODE == 0 ? 0 : i][MODE == 0 ? 0 : j][4 * g + e] =
                fminf(smin[MODE == 0 ? 0 : i][MODE == 0 ? 0 : j][4 * g + e], s);
            acc[i][j][4 * g + e] = 0.f;
          }
        __builtin_amdgcn_sched_barrier(0);
      }
  };

  // ---- main loop: two-stage ring, one barrier per step.  The loads of step u+1 are issued
  // right after the barrier of step u; the last step of a phase issues the first step of the
  // next phase, so the ring never drains between phases.
  auto run_phase = [&](const __amdgpu_buffer_rsrc_t ra, const __amdgpu_buffer_rsrc_t rb, int base,
                       const __amdgpu_buffer_rsrc_t na, const __amdgpu_buffer_rsrc_t nb, int nbase, bool has_next) {
    for (int u = 0; u < sps; u += 2) {
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // my loads of step u are in LDS
      __syncthreads();                                  // everyone's are, and stage 1 is free
      issue(ra, rb, step_off(base, u + 1), sA1, sB1);
      compute(sA0, sB0);
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __syncthreads();
      if (u + 2 < sps)
        issue(ra, rb, step_off(base, u + 2), sA0, sB0);
      else if (has_next)
        issue(na, nb, step_off(nbase, 0), sA0, sB0);
      compute(sA1, sB1);
    }
  };

  load_scales(0);
  issue(resA[0], resB[0], step_off(0, 0), sA0, sB0);
  if (MODE == 0) {
    run_phase(resA[0], resB[0], 0, resA[1], resB[1], 0, true);
    rescale();
    run_phase(resA[1], resB[1], 0, resA[1], resB[1], 0, false);
  } else {
    for (int h = 0; h < p.H; ++h) {
      run_phase(resA[0], resB[0], h * 256, resA[1], resB[1], h * 256, true);
      rescale();
      run_phase(resA[1], resB[1], h * 256, resA[0], resB[0], (h + 1) * 256, h + 1 < p.H);
      finish_head();
      if (h + 1 < p.H) {
        __syncthreads();  // every wave is done with this head's scales
        load_scales(h + 1);
        // the barriers of the next phase make the new scales visible before they are read
      }
    }
  }

  // ---- tile epilogue: scores, dead/tail masking, top-2 per query column
  float best[TQ], second[TQ];
  int bidx[TQ];
#pragma unroll
  for (int j = 0; j < TQ; ++j) {
    best[j] = -INFINITY;
    second[j] = -INFINITY;
    bidx[j] = -1;
  }
  {
    float fq[TQ];
#pragma unroll
    for (int j = 0; j < TQ; ++j) fq[j] = s_fq[wq * WTQ + j * 32 + (lane & 31)];
#pragma unroll
    for (int i = 0; i < TP; ++i)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int row = row_of(i, g);
        const f32x4 fp = *reinterpret_cast<const f32x4*>(&s_fp[row]);
        const f32x4 bias = *reinterpret_cast<const f32x4*>(&s_bias[row]);
#pragma unroll
        for (int j = 0; j < TQ; ++j)
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            float sc;
            if (MODE == 0)
              sc = acc[i][j][4 * g + e] * (fq[j] * fp[e]) + bias[e];
            else
              sc = smin[MODE == 0 ? 0 : i][MODE == 0 ? 0 : j][4 * g + e] + bias[e];
            top2_push(sc, p0 + row + e, best[j], bidx[j], second[j]);
          }
        __builtin_amdgcn_sched_barrier(0);
      }
  }
  // the two half-waves hold interleaved rows of the same columns
#pragma unroll
  for (int j = 0; j < TQ; ++j) {
    const float b2 = __shfl_xor(best[j], 32);
    const int i2 = __shfl_xor(bidx[j], 32);
    const float s2 = __shfl_xor(second[j], 32);
    top2_merge(best[j], bidx[j], second[j], b2, i2, s2);
  }
  if (lane < 32) {
#pragma unroll
    for (int j = 0; j < TQ; ++j) {
      Part t;
      t.best = best[j];
      t.idx = bidx[j];
      t.second = second[j];
      t.pad = 0;
      s_part[wp][wq * WTQ + j * 32 + lane] = t;
    }
  }
  __syncthreads();
  if (tid < BQ && q0 + tid < p.Q) {
    Part t = s_part[0][tid];
#pragma unroll
    for (int w = 1; w < WP; ++w) {
      const Part u = s_part[w][tid];
      top2_merge(t.best, t.idx, t.second, u.best, u.idx, u.second);
    }
    p.part[((long long)l * p.npt + pt) * p.Q + q0 + tid] = t;
  }
#endif
}

namespace {

// Merge the per-pool-tile partial results of every query and take the decision against tau.
__global__ __launch_bounds__(256) void match_finalize_kernel(const Part* __restrict__ part, int npt, long long LQ,
                                                             int Q, float tau, int32_t* __restrict__ best_idx,
                                                             float* __restrict__ best_score,
                                                             int32_t* __restrict__ match_idx,
                                                             float* __restrict__ second_score) {
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= LQ) return;
  const long long l = i / Q, q = i % Q;
  float best = -INFINITY, second = -INFINITY;
  int bidx = -1;
  for (int t = 0; t < npt; ++t) {
    const Part u = part[(l * npt + t) * Q + q];
    top2_merge(best, bidx, second, u.best, u.idx, u.second);
  }
  best_idx[i] = bidx;
  best_score[i] = best;
  match_idx[i] = (bidx >= 0 && best >= tau) ? bidx : -1;
  if (second_score) second_score[i] = second;
}

// Tile shapes.  Block mode keeps a 128x128 accumulator tile per wave (all 256 accumulation
// registers of a lane); per-head-all mode needs a second register tile for the running minimum
// over heads and therefore uses half the rows.
struct TileShape {
  int bp, bq;
};
constexpr TileShape kBlockTile = {256, 256};
constexpr TileShape kHeadTile = {128, 256};

inline TileShape tile_for(int mode) { return mode == RC_SCORE_BLOCK ? kBlockTile : kHeadTile; }

template <bool BF16>
void launch_tiles(int mode, const MatchParams& mp, unsigned grid, hipStream_t st) {
  if (mode == RC_SCORE_BLOCK)
    match_tile_kernel<BF16, kBlockTile.bp, kBlockTile.bq, 2, 2, 0, 1><<<grid, 256, 0, st>>>(mp);
  else
    match_tile_kernel<BF16, kHeadTile.bp, kHeadTile.bq, 2, 2, 1, 1><<<grid, 256, 0, st>>>(mp);
}

}  // namespace
}  // namespace rc

extern "C" size_t rc_match_workspace_size(const rc_kv_desc* qdesc, int32_t mode, int64_t Q, int64_t P) {
  using namespace rc;
  if (!qdesc || Q < 0 || P < 0 || qdesc->n_layers < 0) return 0;
  if (mode != RC_SCORE_BLOCK && mode != RC_SCORE_PER_HEAD_ALL) return 0;
  const TileShape ts = tile_for(mode);
  const int64_t npt = (P + ts.bp - 1) / ts.bp;
  const int64_t n = (int64_t)qdesc->n_layers * (npt > 0 ? npt : 1) * Q;
  return (size_t)(n > 0 ? n : 1) * sizeof(Part);
}

extern "C" rc_status rc_match_blocks(const rc_kv_desc* qdesc, const rc_kv_desc* pdesc, int32_t mode, const void* kq,
                                     const void* vq, int64_t Q, const float* q_ksq, const float* q_vsq,
                                     const void* kp, const void* vp, int64_t P, const float* p_ksq,
                                     const float* p_vsq, const uint8_t* pool_live, float tau, int32_t* best_idx,
                                     float* best_score, int32_t* match_idx, float* second_score, void* workspace,
                                     size_t workspace_bytes, void* hip_stream) {
  using namespace rc;
  clear_error();
  if (rc_status s = check_desc(qdesc, Q, "rc_match_blocks(query)")) return s;
  if (rc_status s = check_desc(pdesc, P, "rc_match_blocks(pool)")) return s;
  if (mode != RC_SCORE_BLOCK && mode != RC_SCORE_PER_HEAD_ALL)
    return fail(RC_ERR_UNSUPPORTED, "rc_match_blocks: mode %d", mode);
  if (qdesc->n_layers != pdesc->n_layers || qdesc->block_tokens != pdesc->block_tokens ||
      qdesc->n_kv_heads != pdesc->n_kv_heads || qdesc->head_dim != pdesc->head_dim || qdesc->dtype != pdesc->dtype)
    return fail(RC_ERR_INVALID_ARG, "rc_match_blocks: query and pool descriptors differ in more than layer_stride");
  if (!(tau == tau)) return fail(RC_ERR_INVALID_ARG, "rc_match_blocks: tau is NaN");
  const int L = qdesc->n_layers;
  if (L == 0 || Q == 0) return RC_OK;
  if (!kq || !vq || !q_ksq || !q_vsq || !best_idx || !best_score || !match_idx)
    return fail(RC_ERR_INVALID_ARG, "rc_match_blocks: NULL query or output pointer");
  if (P > 0 && (!kp || !vp || !p_ksq || !p_vsq)) return fail(RC_ERR_INVALID_ARG, "rc_match_blocks: NULL pool pointer");
  if (!aligned16(kq) || !aligned16(vq) || !aligned16(kp) || !aligned16(vp))
    return fail(RC_ERR_INVALID_ARG, "rc_match_blocks: KV pointer not 16-byte aligned");
  const TileShape ts = tile_for(mode);
  const int64_t npt = (P + ts.bp - 1) / ts.bp, nqt = (Q + ts.bq - 1) / ts.bq;
  const int64_t total = (int64_t)L * npt * nqt;
  if (Q > 0x7fffffffLL || P > 0x7fffffffLL || total > 0x3fffffffLL || (int64_t)L * Q > 0x7fffffffLL * 128)
    return fail(RC_ERR_UNSUPPORTED, "rc_match_blocks: problem beyond the grid limits");
  const size_t need = rc_match_workspace_size(qdesc, mode, Q, P);
  if (!workspace || workspace_bytes < need || !aligned16(workspace))
    return fail(RC_ERR_WORKSPACE, "rc_match_blocks: workspace of %zu bytes needed (16-byte aligned), got %zu", need,
                workspace_bytes);
  hipStream_t st = static_cast<hipStream_t>(hip_stream);

  if (P > 0) {
    MatchParams mp;
    mp.kq = static_cast<const char*>(kq);
    mp.vq = static_cast<const char*>(vq);
    mp.kp = static_cast<const char*>(kp);
    mp.vp = static_cast<const char*>(vp);
    mp.q_ksq = q_ksq;
    mp.q_vsq = q_vsq;
    mp.p_ksq = p_ksq;
    mp.p_vsq = p_vsq;
    mp.live = pool_live;
    mp.part = static_cast<Part*>(workspace);
    mp.q_lstride_b = qdesc->layer_stride * 2;
    mp.p_lstride_b = pdesc->layer_stride * 2;
    mp.L = L;
    mp.Q = (int)Q;
    mp.P = (int)P;
    mp.T = qdesc->block_tokens;
    mp.H = qdesc->n_kv_heads;
    mp.npt = (int)npt;
    mp.nqt = (int)nqt;
    mp.total = (int)total;
    mp.chunk = 32;
    const int64_t per_round = 8LL * mp.chunk;
    const unsigned grid = (unsigned)(((total + per_round - 1) / per_round) * per_round);
    if (qdesc->dtype == RC_BF16)
      launch_tiles<true>(mode, mp, grid, st);
    else
      launch_tiles<false>(mode, mp, grid, st);
    if (rc_status s = check_launch("rc_match_blocks(tiles)")) return s;
  }
  const long long LQ = (long long)L * Q;
  match_finalize_kernel<<<(unsigned)((LQ + 255) / 256), 256, 0, st>>>(static_cast<const Part*>(workspace), (int)npt, LQ,
                                                                     (int)Q, tau, best_idx, best_score, match_idx,
                                                                     second_score);
  return check_launch("rc_match_blocks(finalize)");
}
