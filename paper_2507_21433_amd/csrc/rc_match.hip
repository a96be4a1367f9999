// rc_match_blocks: query-block x pool-block score contraction on the matrix cores with a fused
// top-1 / runner-up / threshold selection (ReasonCache Sec. IV-A Stage 2: with the squared norms
// cached, comparing two blocks only needs the dot product of the flattened tensors).
//
// Shape of the work per layer: S[P x Q] = Xp[P x D] * Xq[Q x D]^T for the K tensors and again for
// the V tensors; both operands are contiguous along the reduction dimension.  Pool blocks are the
// rows of the MFMA tile (they land in the accumulator registers of a lane), query blocks are the
// columns (they land on lanes), so the argmax over the pool is mostly an in-lane reduction.
//
// One workgroup (4 waves, one per SIMD) owns a BP x BQ tile of S for the whole reduction (no
// split-K, so the selection can be fused); each wave holds a (BP/2) x (BQ/2) accumulator tile.
// Operand slices of 64 elements (128 bytes per block, one L2 line) go global -> LDS with
// direct-to-LDS 16-byte buffer loads.  With a 256 x 256 tile all of the 160 KB of LDS is ring
// buffer: three stages for the pool slices (two always in flight) and two for the query slices,
// which come from the L2.  In the steady-state loop a matrix instruction is in flight 95 % of
// the time (a wave issues one instruction every four cycles, a 32x32x16 matrix instruction takes
// 32, and the loads, LDS reads and bookkeeping of a step are placed in the issue slots between);
// what bounds the launch then is the clock: under this load the chip runs at about 1.5 GHz, not
// the 2.4 GHz of its peak figure, and each XCD at a clock of its own.  The 16-byte chunks of an
// LDS row are XOR-swizzled by the row number so that fragment reads spread over all banks.
//
// The same kernel body serves three modes: the cosine score per layer (MODE 0), the same per KV
// head with the minimum over heads (MODE 1), and the layer-mean Euclidean distance of the
// paper's block-distance equation, for which a workgroup walks a group of layers (MODE 2).
//
// K and V are normalised by different norms but share one accumulator tile: after the K
// phase the accumulators are multiplied by (aKq aKp)/(aVq aVp), the V phase continues into
// them, and the epilogue multiplies by aVq aVp / 2, with a = 1/sqrt(squared norm).
#include <hip/hip_runtime.h>

#include <type_traits>

#include "rc_common.hpp"

namespace rc {
namespace {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef short i16x2 __attribute__((ext_vector_type(2)));

// Two scores in [-1, 1] onto the grid of 1/32767 (signed normalised 16 bit, round to nearest).  The
// per-head-all mode keeps its minimum over heads on this grid; both of its paths call this.
__device__ __forceinline__ i16x2 quantise_pair(float a, float b) { return __builtin_amdgcn_cvt_pknorm_i16(a, b); }

constexpr int kBK = 64;             // reduction elements per pipeline step
constexpr int kRowBytes = kBK * 2;  // bytes of one block's slice in LDS (one 128-byte line)
constexpr int kPoolWaves = 2, kQueryWaves = 2;  // waves of a workgroup along the two tile sides
constexpr int kThreads = 64 * kPoolWaves * kQueryWaves;
constexpr int kMaxGrid = 512;                          // workgroups of a tile-kernel launch, at most
constexpr int kScheduleHeader = (8 + kMaxGrid) * 32;   // ints ahead of the claim words of a dynamic tile schedule
constexpr int kPoolStages = 3, kQueryStages = 2;

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
  Part* part;                          // [L][npt][Q]
  float* dpart;                        // layer-mean mode: [groups][P][Q] sums of layer distances
  long long q_lstride_b, p_lstride_b;  // bytes between layers
  int L, Q, P;
  int T, H;
  int npt, nqt;
  int total;  // L * npt * nqt (layer-mean mode: groups * npt * nqt)
  int vgrid;  // virtual workgroups: total rounded up to whole rounds of 8 XCDs x chunk; the launch walks them
  int* ctr;        // nullptr = a fixed schedule; else zero at launch: 8 counters of slots taken from a list's back, one
                   // progress word per workgroup (each on 128 bytes of its own), then from [kScheduleHeader] on the
                   // claim words, `rounds` of them per workgroup
  int rounds;      // slots in one workgroup's walk
  int dyn_from;    // slots from this one on can be taken from the back of their list
  int steal_min;   // a slot is taken from a list's back only if its own workgroup is at least this far short of it
  int raw;    // MODE 3: the shares hold the bare dot products (the layer-mean distance is formed from their sums)
  int chunk;  // tiles handed to one XCD in a row
  int G;      // layer-mean mode: layers per group (one workgroup walks the layers of its group)
  int S;      // split mode: workgroups per tile, each over its own part of the reduction (even)
  int stagger_wgs;   // workgroups of the first round (one per compute unit) ...
  int stagger_unit;  // ... start (tile % 16) * stagger_unit * 1024 clocks late
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

// From the squared norms of a block's K and V tensors: ratio = aK/aV and av = aV with
// a = 1/sqrt(squared norm).  A zero K norm gives aK = 0 (cosine defined as 0); a zero V norm
// gives aV = 1, which is harmless because every V dot product of that block is 0 as well.
// v_rsq_f32 is good to 1 ulp; the scores only need 2e-3.
__device__ __forceinline__ void norm_factors(float ksq, float vsq, float& ratio, float& av) {
  const float ak = ksq > 0.f ? __builtin_amdgcn_rsqf(ksq) : 0.f;
  av = vsq > 0.f ? __builtin_amdgcn_rsqf(vsq) : 1.f;
  const float inv_av = vsq > 0.f ? vsq * av : 1.f;  // sqrt(vsq)
  ratio = ak * inv_av;
}

// Raw buffer descriptor (base, no stride, byte range, 32-bit raw data format) in scalar registers.
__device__ __forceinline__ i32x4 make_srd(const void* base, uint32_t bytes) {
  const unsigned long long a = (unsigned long long)base;
  i32x4 r;
  r[0] = __builtin_amdgcn_readfirstlane((int)(uint32_t)a);
  r[1] = __builtin_amdgcn_readfirstlane((int)((a >> 32) & 0xffffu));
  r[2] = __builtin_amdgcn_readfirstlane((int)bytes);
  r[3] = 0x00020000;
  return r;
}

// 16 bytes per lane, global -> LDS without passing through registers: lane l lands at LDS byte
// lds_base + 16*l.  Completion is counted by vmcnt, in issue order.  Written as asm so that the
// pipeline's waits are exactly the ones placed by hand below.
// STREAM marks the load non-temporal: the pool slices are read once (or by the few query tiles of
// the same pool tile, close together in time), so they should not displace the query slices that
// every pool tile of the layer re-reads from the L2.  Measured: 2.5 % on cfg2, 1.5 % on cfg3.
template <bool STREAM>
__device__ __forceinline__ void dma16(i32x4 srd, uint32_t voff, uint32_t soff, uint32_t lds_base) {
  // the descriptor, the scalar offset and the LDS base are the same for the whole wave
  srd[0] = __builtin_amdgcn_readfirstlane(srd[0]);
  srd[1] = __builtin_amdgcn_readfirstlane(srd[1]);
  srd[2] = __builtin_amdgcn_readfirstlane(srd[2]);
  srd[3] = __builtin_amdgcn_readfirstlane(srd[3]);
  soff = __builtin_amdgcn_readfirstlane(soff);
  lds_base = __builtin_amdgcn_readfirstlane(lds_base);
  if (STREAM)
    asm volatile("s_mov_b32 m0, %3\n\ts_nop 0\n\tbuffer_load_dwordx4 %0, %1, %2 offen nt lds"
                 :
                 : "v"(voff), "s"(srd), "s"(soff), "s"(lds_base)
                 : "memory", "m0");
  else
    asm volatile("s_mov_b32 m0, %3\n\ts_nop 0\n\tbuffer_load_dwordx4 %0, %1, %2 offen lds"
                 :
                 : "v"(voff), "s"(srd), "s"(soff), "s"(lds_base)
                 : "memory", "m0");
}

__device__ __forceinline__ uint32_t lds_offset(const void* p) {
  return (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) char*)p;
}

// Position in the reduction: phase ph (tensor = ph & 1, head = ph >> 1), step u of the phase.
struct Cursor {
  int u, ph;
};

}  // namespace

// BP x BQ tile of one layer.  MODE 0 = block score, 1 = per-head-all, 2 = layer-mean Euclidean
// distance (the tile of a group of layers: the workgroup walks the layers one after the other and
// adds |Kq-Kp| + |Vq-Vp| of every layer to the tile's running sum), 3 = block score of a problem
// with too few tiles to fill the chip: S workgroups share a tile, each takes 1/(S/2) of the K or of
// the V reduction and stores its share of the scores, (aKq aKp <Kq,Kp>)/2 or (aVq aVp <Vq,Vp>)/2
// over its elements, as a 256x256 tile of floats; a second kernel adds the S shares and selects.
// MODE 4 = the same for the per-head-all score: S = H shares, share h computes the score of head h
// over the head's K and V slices, and the second kernel takes the minimum over the shares.
// SHARED_POOL: several query tiles, i.e. several workgroups read every pool slice (see the pool loads below).
template <bool BF16, int BP, int BQ, int MODE, bool SHARED_POOL = false>
__global__ __launch_bounds__(kThreads, 1) void match_tile_kernel(const MatchParams p) {
#if defined(__HIP_DEVICE_COMPILE__)  // the host pass only needs the launch stub
  constexpr int NT = kThreads, WP = kPoolWaves, WQ = kQueryWaves;
  constexpr int WTP = BP / WP, WTQ = BQ / WQ;
  constexpr int TP = WTP / 32, TQ = WTQ / 32;
  constexpr int LA = BP * 8 / NT, LB = BQ * 8 / NT;  // 16-byte loads per thread per step
  constexpr int SA = kPoolStages, SB = kQueryStages;
  constexpr int A_STAGE = BP * kRowBytes, B_STAGE = BQ * kRowBytes;
  constexpr int RING = SA * A_STAGE + SB * B_STAGE;
  static_assert(BP % (32 * WP) == 0 && BQ % (32 * WQ) == 0, "wave tiles are multiples of 32");
  static_assert(NT >= BQ, "one thread per query column in the tile epilogue");
  static_assert(RING <= 160 * 1024, "ring fits the LDS of a compute unit");
  static_assert(sizeof(Part) * WP * BQ <= RING, "the epilogue scratch reuses the ring");
  static_assert(MODE < 2 || (BP == 256 && BQ == 256 && WP == 2 && WQ == 2), "sum_index() decodes this tile shape");
  constexpr bool SHARES = (MODE == 3 || MODE == 4);    // several workgroups per tile, results stored as tiles of floats
  constexpr bool PER_HEAD = (MODE == 1 || MODE == 4);  // phases are heads' [T][Dh] slices, norms are per head

  __shared__ __attribute__((aligned(1024))) char s_ring[RING];
  const uint32_t ringA = lds_offset(s_ring), ringB = ringA + SA * A_STAGE;

  // ---- which tiles: the launch has one workgroup per compute unit, each walks tiles of a grid of
  // p.vgrid virtual workgroups.  Virtual workgroup v belongs to XCD v & 7, and consecutive runs of
  // `chunk` tiles go to one XCD, so tiles that share operands share an L2.  The virtual workgroups form 8
  // lists, one per XCD, of p.vgrid / 8 slots each; workgroup b walks list b & 7 from slot b >> 3 in strides
  // of gridDim.x / 8.  With a fixed schedule (p.ctr == nullptr) that is all.
  // The XCDs of one chip run this kernel at clocks of their own (measured: 8 % between the fastest and the
  // slowest on one box), so with many rounds the fast ones would idle at the end.  Then the slots from
  // p.dyn_from on (the tail of every list) have a claim word each, and a workgroup owns such a slot only once it
  // has swapped that word from 0 to 1; the slots before are walked as in the fixed schedule (a swap per tile
  // costs more than the scheme gains: measured 4 % of the launch with every slot claimed).  The walk stays as it is
  // (the workgroups that share a pool tile keep running side by side and find each other's slices in the L2:
  // handing tiles out in order of arrival costs 3 % with several query tiles), but a workgroup that is through
  // with it takes slots from the BACK of the list whose workgroups are furthest behind.  A tile taken that way
  // ends a whole tile time later, so it is taken only if the workgroup whose walk contains it is at least
  // p.steal_min slots short of it (every workgroup publishes the slot it works on).  A walk skips what was
  // taken.  All of this is words that one workgroup writes or swaps at a time, on cache lines of their own:
  // counters that all workgroups add to cost more than the scheme gains.  Which workgroup computes a tile does
  // not change the tile's result.
  const bool dynamic = p.ctr != nullptr;
  const int nslots = p.vgrid >> 3;
  const int my_list = blockIdx.x & 7, my_pos = blockIdx.x >> 3, stride = gridDim.x >> 3;
  // the claim words of one workgroup's walk lie together: [list][position][round]
  auto claim_of = [&](int list, int slot) { return p.ctr + kScheduleHeader + (list * stride + slot % stride) * p.rounds + slot / stride; };
  auto progress_of = [&](int list, int pos) { return p.ctr + (8 + list * stride + pos) * 32; };
  auto taken_of = [&](int list) { return p.ctr + list * 32; };
  // Thread 0 keeps the walk: my_slot, and what its claim word held before this workgroup's swap (0 = the slot
  // is this workgroup's).  The swap for the next slot of the walk goes out when a tile's last phase ends and is
  // looked at after the tile's epilogue, so nobody waits for it (and no steady-state loop runs with its answer
  // pending).
  int my_slot = my_pos, prev = 1;
  bool walking = dynamic && my_slot < nslots, home_tile = false;
  // slots ahead of p.dyn_from are never taken from the back and need no claim
  auto claim = [&](int slot) { return slot < p.dyn_from ? 0 : atomicExch(claim_of(my_list, slot), 1); };
  if (walking && threadIdx.x == 0) prev = claim(my_slot);
  auto claim_next = [&]() __attribute__((always_inline)) {
    if (dynamic && threadIdx.x == 0 && home_tile) {
      my_slot += stride;
      walking = my_slot < nslots;
      prev = 1;
      if (walking) prev = claim(my_slot);
    }
  };
  for (int round = 0;; ++round) {
  // every wave is done with the ring (last fragments, epilogue scratch) before the next tile's loads land in it
  if (round) __syncthreads();
  int wg;
  if (dynamic) {
    volatile int* box = reinterpret_cast<volatile int*>(s_ring);  // the ring is free between tiles
    if (threadIdx.x == 0) {
      int slot = -1, list = my_list;
      while (walking && prev != 0) {  // taken from the back by another workgroup: on to the next slot of the walk
        my_slot += stride;
        walking = my_slot < nslots;
        if (walking) prev = claim(my_slot);
      }
      home_tile = walking;
      if (walking) {
        slot = my_slot;
        if (slot + 2 * stride >= p.dyn_from)
          __hip_atomic_store(progress_of(my_list, my_pos), slot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      } else {
        unsigned closed = 1u << my_list;
        for (int tries = 0; tries < 16 && slot < 0; ++tries) {
          int least = 0x7fffffff;
          list = -1;
          for (int x = 0; x < 8; ++x) {
            if (closed >> x & 1) continue;
            const int at = __hip_atomic_load(progress_of(x, my_pos), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (at < least) { least = at; list = x; }
          }
          if (list < 0) break;
          const int from_back = nslots - 1 - atomicAdd(taken_of(list), 1);
          const int at = from_back < p.dyn_from ? 0x7fffffff
                                       : __hip_atomic_load(progress_of(list, from_back % stride), __ATOMIC_RELAXED,
                                                           __HIP_MEMORY_SCOPE_AGENT);
          if (from_back < p.dyn_from || from_back - at < p.steal_min)
            closed |= 1u << list;  // the list's own workgroups are about to reach its back
          else if (atomicExch(claim_of(list, from_back), 1) == 0)
            slot = from_back;
        }
      }
      box[0] = slot;
      box[1] = list;
    }
    __syncthreads();
    const int slot_d = __builtin_amdgcn_readfirstlane(box[0]);
    const int list_d = __builtin_amdgcn_readfirstlane(box[1]);
    __syncthreads();
    if (slot_d < 0) break;  // nothing left that is worth taking
    wg = slot_d * 8 + list_d;
  } else {
    wg = blockIdx.x + round * gridDim.x;
    if (wg >= p.vgrid) break;
  }
  const int slot = wg >> 3;
  const int tile = ((slot / p.chunk) * 8 + (wg & 7)) * p.chunk + slot % p.chunk;
  if (tile >= p.total) {
    claim_next();
    continue;
  }
  const int split = SHARES ? tile % p.S : 0;   // which share of the tile (MODE 3: part of the reduction, MODE 4: head)
  const int tile_id = SHARES ? tile / p.S : tile;
  const int qt = tile_id % p.nqt;
  const int pt = (tile_id / p.nqt) % p.npt;
  const int lz = tile_id / (p.nqt * p.npt);  // layer, or group of layers in mode 2
  const int l_first = (MODE == 2) ? lz * p.G : lz;
  const int nl = (MODE == 2) ? min(p.G, p.L - l_first) : 1;
  int l = l_first;
  const int p0 = pt * BP, q0 = qt * BQ;

  // The tiles that run on one XCD at the same time read the same query slices (and, with several
  // query tiles, the same pool slices).  Started together they ask the L2 for the same lines at
  // the same moment, step after step.  The workgroups of the first round therefore start spread
  // in time by the position of their pool tile within the XCD's run of tiles (the query tiles of
  // one pool tile stay together: the second one finds the pool slice in the L2 only if it follows
  // closely); later rounds inherit the spread.  Nothing else changes.  Measured on one box against
  // an unspread start: 3 % faster with one query tile (Q = 256), 5 % in per-head mode (Q = 512),
  // within 0.5 % with four query tiles (Q = 1024).
  if (round == 0 && (int)blockIdx.x < p.stagger_wgs)
    for (int i = 0; i < (((slot % p.chunk) / p.nqt) & 15) * p.stagger_unit; ++i) __builtin_amdgcn_s_sleep(16);

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wp = wave / WQ, wq = wave % WQ;

  const int D = p.T * p.H * 128;
  const long long row_b = (long long)D * 2;
  const int rowsA = min(BP, p.P - p0), rowsB = min(BQ, p.Q - q0);

  // ---- buffer descriptors over this tile's rows of the four tensors.  The range check of the
  // buffer unit is a second guard; offsets are kept inside the rows anyway.
  i32x4 srdAk, srdAv, srdBk, srdBv;
  auto set_layer_tensors = [&]() {
    const long long offPool = l * p.p_lstride_b + (long long)p0 * row_b;
    const long long offQry = l * p.q_lstride_b + (long long)q0 * row_b;
    srdAk = make_srd(p.kp + offPool, (uint32_t)(rowsA * row_b));
    srdAv = make_srd(p.vp + offPool, (uint32_t)(rowsA * row_b));
    srdBk = make_srd(p.kq + offQry, (uint32_t)(rowsB * row_b));
    srdBv = make_srd(p.vq + offQry, (uint32_t)(rowsB * row_b));
  };
  set_layer_tensors();

  // ---- LDS layout of a stage: row r (one block) holds its 128-byte slice as eight 16-byte
  // chunks; logical chunk c sits at physical chunk c ^ (r & 7).  A fragment read (32 consecutive
  // rows, chunks 2kk and 2kk+1) then runs at the full LDS rate (measured: 110 B/clk per compute
  // unit, against 32 B/clk for the unswizzled layout).
  // Load i of a wave fills rows (i*NT + wave*64)/8 .. +7; lane -> (row lane/8, physical chunk
  // lane%8).  The lane's byte offset for load 0 is a register, the row step of load i (32 rows)
  // goes into the scalar offset.  Rows past the end of the pool / queries fall outside the
  // descriptor's range and read as zeros (their results are masked anyway).
  const int rho = lane >> 3;
  const uint32_t src_chunk = (uint32_t)(((lane & 7) ^ rho) * 16);
  const uint32_t voff = (uint32_t)(tid >> 3) * (uint32_t)row_b + src_chunk;
  const uint32_t load_stride = (uint32_t)(NT / 8) * (uint32_t)row_b;

  // fragment reads: lane -> row lane%32 of a 32-row group, logical chunk 2*kk + lane/32
  const uint32_t sw = (uint32_t)(lane & 7);
  const uint32_t fragA = (uint32_t)((wp * WTP + (lane & 31)) * kRowBytes);
  const uint32_t fragB = (uint32_t)((wq * WTQ + (lane & 31)) * kRowBytes);

  // ---- steps.  A phase is one tensor (K or V) of the whole block (MODE 0) or of one head
  // (MODE 1).  Step u of a phase reads 128 bytes per block at byte offset
  // head*256 + (u/2)*tok + (u%2)*128:  tok = 256 walks the flattened block, tok = H*256 walks
  // one head's [T][Dh] slice.
  // MODE 3: one phase of (D/kBK)/(S/2) steps, starting at step u_first of the K tensor (shares
  // 0 .. S/2-1) or of the V tensor (the others).
  // MODE 4: the two phases of head `split`, i.e. phases 2*split and 2*split + 1 of MODE 1.
  const int sps = (MODE == 3) ? (D / kBK) / (p.S / 2) : !PER_HEAD ? (D / kBK) : (p.T * 2);
  const int nphase = (MODE == 3) ? 1 : (MODE == 4) ? 2 * split + 2 : !PER_HEAD ? 2 : 2 * p.H;
  const int ph_first = (MODE == 4) ? 2 * split : 0;
  const int tok = !PER_HEAD ? 256 : p.H * 256;
  const bool split_v = (MODE == 3) && split >= p.S / 2;
  const int u_first = (MODE == 3) ? (split % (p.S / 2)) * sps : 0;
  auto advance = [&](Cursor& c) {
    if (++c.u == sps) {
      c.u = 0;
      ++c.ph;
    }
  };
  auto byte_off = [&](const Cursor& c) {
    if (MODE == 3) return (uint32_t)((c.u + u_first) * 128);
    return (uint32_t)((c.ph >> 1) * 256 + (c.u >> 1) * tok + (c.u & 1) * 128);
  };

  // Where the next pool / query slice comes from and which ring stage it goes to.  Past the last
  // step the cursor stays on the last slice: the two refills that nobody needs re-read valid
  // data, so every step issues the same number of loads and the wait counts stay uniform.
  struct Feed {
    Cursor cur;
    int stage;
    i32x4 srd;
    uint32_t off, dst;
  };
  Feed fa{{0, ph_first}, 0, srdAk, 0, 0}, fb{{0, ph_first}, 0, srdBk, 0, 0};
  auto prepare_src = [&](Feed& f, const i32x4& k_srd, const i32x4& v_srd) {
    f.srd = ((MODE == 3) ? split_v : (f.cur.ph & 1) != 0) ? v_srd : k_srd;
    f.off = byte_off(f.cur);
  };
  auto prepare_dst = [&](Feed& f, uint32_t ring, int stage_bytes) { f.dst = ring + f.stage * stage_bytes + wave * 1024; };
  auto prepare = [&](Feed& f, const i32x4& k_srd, const i32x4& v_srd, uint32_t ring, int stage_bytes) {
    prepare_src(f, k_srd, v_srd);
    prepare_dst(f, ring, stage_bytes);
  };
  // the next slice of the same phase: the cursor counts on and the offset follows (same tensor)
  auto bump = [&](Feed& f) {
    if (PER_HEAD)
      f.off += (f.cur.u & 1) ? (uint32_t)(tok - 128) : 128u;
    else
      f.off += 128u;
    ++f.cur.u;
  };
  auto move_cursor = [&](Feed& f) {
    Cursor n = f.cur;
    advance(n);
    if (n.ph < nphase) f.cur = n;
  };
  auto next_stage = [&](Feed& f, int stages) { f.stage = (f.stage + 1 == stages) ? 0 : f.stage + 1; };
  auto next = [&](Feed& f, int stages) {
    move_cursor(f);
    next_stage(f, stages);
  };
  // The pool loads carry the non-temporal hint when nobody else reads the slice (one query tile, cfg2: 8 % less
  // launch time than without it, since the slice then does not displace the query slices that every pool tile
  // of the layer re-reads from the L2).  With several query tiles the workgroups that share a pool tile want to
  // find each other's slice in the L2, and a line that is not kept can be gone before the last of them asks for
  // it: 0.5-1.4 % on the Q = 1024 workloads, and in the layer-mean mode, where those workgroups leave a fold
  // (a read-modify-write of 256 KB each) a few microseconds apart, twice the L2-out traffic and 6 % of the
  // launch.  The cosine mode is compiled in both forms, the layer-mean mode without the hint; the per-head and
  // the few-tiles modes keep it (measured: no difference there).
  auto dmaA = [&](int i) {
    dma16<MODE != 2 && !SHARED_POOL>(fa.srd, voff, fa.off + i * load_stride, fa.dst + i * NT * 16);
  };
  auto dmaB = [&](int i) { dma16<false>(fb.srd, voff, fb.off + i * load_stride, fb.dst + i * NT * 16); };

  f32x16 acc[TP][TQ];
#pragma unroll
  for (int i = 0; i < TP; ++i)
#pragma unroll
    for (int j = 0; j < TQ; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // One step = 4 sub-steps of 16 reduction elements = 4 batches of TP*TQ matrix instructions.
  //  - Fragments of a sub-step are requested one batch before they are multiplied.
  //  - The last batch of a step is issued after the next step's barrier: its fragments are
  //    already in registers, so the matrix cores have work while the first fragment reads of
  //    the new step are in flight.
  //  - The step's LB + LA refill loads are spread between the matrix instructions (query slice
  //    first): the texture unit takes a 1 KB wave load every 16 cycles, and a wave that issues
  //    its loads in one burst sits in that queue instead of feeding the matrix cores.
  // The scheduling barriers pin this order.
  constexpr int SLOTS = 4 * TP, LPS = (LA + LB + SLOTS - 1) / SLOTS;
  // One batch = the TP*TQ matrix instructions of a sub-step, row tile by row tile.  Between the
  // instructions of row tile i ride the reads of the next sub-step's fragments that belong to it
  // (A fragment i behind the first instruction, B fragment i behind the last) and the row's
  // share of the refill loads (in the middle): LDS reads and loads are spread evenly over the
  // step instead of arriving in bursts right after the barrier, when all four waves would ask
  // the LDS for 8 KB each at the same moment.  Measured on one box against a burst of eight
  // reads per sub-step: 5-7 % on the Q = 1024 workloads, 3-4 % in per-head mode, 1-2 % on cfg2.
  // The scalar bookkeeping of the two feeds (which slice comes next, from which tensor, into which
  // ring stage) and of the read stages rides in those rows too (`slot_work`), a few instructions per
  // row, in the gap behind the instruction after the load's.  A wave issues one instruction every
  // four cycles and a matrix instruction covers seven more issues; left at the end of the step the
  // bookkeeping sits between the last matrix instruction of one step and the first of the next,
  // some thirty scalar instructions with nothing to hide behind (measured: 200 of the 2400 cycles
  // of a step).  Slot s is row s % TP of batch s / TP; the query loads are slots 0 .. LB-1, the
  // pool loads slots LB .. LB+LA-1.  The pool feed moves on just before its loads, the query feed
  // after its loads (for the next step), then the read stages of the next step.
  // FAST steps are those whose two feeds stay inside the phase (all but the last two of a phase):
  // the cursor just counts and the tensor does not change; the last two steps take the general code.
  static_assert(TQ <= TP, "B fragment j is read behind row tile j");
  static_assert(LPS == 1 && LB >= 2 && LB + 3 < SLOTS, "one load per slot, and room for the bookkeeping slots");
  int rdA = 0, rdB = 0;                   // ring stages the current step reads
  const char *sA_next = s_ring, *sB_next = s_ring + SA * A_STAGE;
  constexpr int W0 = LB >= 3 ? LB - 3 : 0;  // first bookkeeping slot
  auto slot_work = [&](auto fast_tag, int slot) __attribute__((always_inline)) {
    constexpr bool FAST = decltype(fast_tag)::value;
    // pool feed: cursor, then stage and destination, then (general code) tensor and offset: ready before slot LB
    if (slot == W0) {
      if (FAST) bump(fa); else move_cursor(fa);
    }
    if (slot == (LB >= 3 ? W0 + 1 : W0)) {
      next_stage(fa, SA);
      prepare_dst(fa, ringA, A_STAGE);
    }
    if (slot == LB - 1 && !FAST) prepare_src(fa, srdAk, srdAv);
    // query feed, for the loads of the next step
    if (slot == LB) {
      if (FAST) bump(fb); else move_cursor(fb);
    }
    if (slot == LB + (LB >= 3 ? 1 : 0)) {
      next_stage(fb, SB);
      prepare_dst(fb, ringB, B_STAGE);
    }
    if (slot == LB + (LB >= 3 ? 2 : 1) && !FAST) prepare_src(fb, srdBk, srdBv);
    if (slot == LB + (LB >= 3 ? 3 : 2)) {
      rdA = (rdA + 1 == SA) ? 0 : rdA + 1;
      rdB = (rdB + 1 == SB) ? 0 : rdB + 1;
      sA_next = s_ring + rdA * A_STAGE;
      sB_next = s_ring + SA * A_STAGE + rdB * B_STAGE;
    }
  };
  auto batch = [&](auto fast_tag, const uint4 (&af)[TP], const uint4 (&bf)[TQ], int b, const char* sA, const char* sB,
                   int kk, uint4 (&naf)[TP], uint4 (&nbf)[TQ]) __attribute__((always_inline)) {
    const uint32_t c = (((uint32_t)(2 * kk) + (uint32_t)(lane >> 5)) ^ sw) * 16;
    constexpr int JD = TQ > 1 ? TQ / 2 - 1 : 0;  // the refill load follows this instruction of the row ...
    constexpr int JW = TQ > 2 ? JD + 1 : JD;     // ... the bookkeeping the next one, where the row has a gap to spare
#pragma unroll
    for (int i = 0; i < TP; ++i) {
#pragma unroll
      for (int j = 0; j < TQ; ++j) {
        acc[i][j] = mfma<BF16>(af[i], bf[j], acc[i][j]);
        if (j == 0) {
          naf[i] = *reinterpret_cast<const uint4*>(sA + fragA + i * 32 * kRowBytes + c);
          __builtin_amdgcn_sched_barrier(0);
        }
        if (j == JD) {
#pragma unroll
          for (int t = 0; t < LPS; ++t) {
            const int n = (b * TP + i) * LPS + t;
            if (n < LB)
              dmaB(n);
            else if (n < LB + LA)
              dmaA(n - LB);
          }
          __builtin_amdgcn_sched_barrier(0);
        }
        if (j == JW) {
          slot_work(fast_tag, b * TP + i);
          __builtin_amdgcn_sched_barrier(0);
        }
        if (j == TQ - 1 && i < TQ) nbf[i < TQ ? i : 0] = *reinterpret_cast<const uint4*>(sB + fragB + i * 32 * kRowBytes + c);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  uint4 fwA[TP], fwB[TQ];  // fragments of the previous step's last sub-step, not multiplied yet
  auto clear_pending = [&]() {
#pragma unroll
    for (int i = 0; i < TP; ++i) fwA[i] = make_uint4(0, 0, 0, 0);
#pragma unroll
    for (int j = 0; j < TQ; ++j) fwB[j] = make_uint4(0, 0, 0, 0);
  };
  auto compute = [&](auto fast_tag, const char* sA, const char* sB) __attribute__((always_inline)) {
    uint4 fa0[TP], fb0[TQ], fa1[TP], fb1[TQ];
    batch(fast_tag, fwA, fwB, 0, sA, sB, 0, fa0, fb0);  // previous step's sub-step 3 (zeros at the start of a phase); reads sub-step 0
    batch(fast_tag, fa0, fb0, 1, sA, sB, 1, fa1, fb1);
    batch(fast_tag, fa1, fb1, 2, sA, sB, 2, fa0, fb0);
    batch(fast_tag, fa0, fb0, 3, sA, sB, 3, fwA, fwB);  // sub-step 3 is multiplied in the next step
  };
  // multiply what is still pending (end of a phase); no refills ride on these instructions
  auto drain = [&]() {
#pragma unroll
    for (int i = 0; i < TP; ++i)
#pragma unroll
      for (int j = 0; j < TQ; ++j) acc[i][j] = mfma<BF16>(fwA[i], fwB[j], acc[i][j]);
  };

  // ---- scale factors, read from the cached squared norms when a phase ends.  Range-checked
  // buffer loads with 32-bit offsets: a row past the end of the pool / queries reads 0.
  const int nh = !PER_HEAD ? 1 : p.H;
  __amdgpu_buffer_rsrc_t nQk, nQv, nPk, nPv;
  auto set_layer_norms = [&]() {
    nQk = __builtin_amdgcn_make_buffer_rsrc((void*)(p.q_ksq + (long long)l * p.Q * nh), 0, p.Q * nh * 4, 0x00020000);
    nQv = __builtin_amdgcn_make_buffer_rsrc((void*)(p.q_vsq + (long long)l * p.Q * nh), 0, p.Q * nh * 4, 0x00020000);
    nPk = __builtin_amdgcn_make_buffer_rsrc((void*)(p.p_ksq + (long long)l * p.P * nh), 0, p.P * nh * 4, 0x00020000);
    nPv = __builtin_amdgcn_make_buffer_rsrc((void*)(p.p_vsq + (long long)l * p.P * nh), 0, p.P * nh * 4, 0x00020000);
  };
  set_layer_norms();
  // Query column j of this lane: ratio rq = aK/aV and final factor fq = aV/2.
  auto query_scales = [&](int head, float (&rq)[TQ], float (&fq)[TQ]) {
#pragma unroll
    for (int j = 0; j < TQ; ++j) {
      const int o = ((q0 + wq * WTQ + j * 32 + (lane & 31)) * nh) * 4;
      const float ksq = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(nQk, o, head * 4, 0));
      const float vsq = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(nQv, o, head * 4, 0));
      float av;
      norm_factors(ksq, vsq, rq[j], av);
      fq[j] = 0.5f * av;
    }
  };
  // Pool rows row .. row+3 of the tile: ratio rp = aK/aV and final factor fp = aV.
  auto pool_scales = [&](int row, int head, f32x4& rp, f32x4& fp) {
    f32x4 ksq, vsq;
    if (!PER_HEAD) {
      typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
      ksq = __builtin_bit_cast(f32x4, (u32x4_t)__builtin_amdgcn_raw_buffer_load_b128(nPk, (p0 + row) * 4, 0, 0));
      vsq = __builtin_bit_cast(f32x4, (u32x4_t)__builtin_amdgcn_raw_buffer_load_b128(nPv, (p0 + row) * 4, 0, 0));
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int o = (p0 + row + e) * nh * 4;
        ksq[e] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(nPk, o, head * 4, 0));
        vsq[e] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(nPv, o, head * 4, 0));
      }
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      float ratio, av;
      norm_factors(ksq[e], vsq[e], ratio, av);
      rp[e] = ratio;
      fp[e] = av;
    }
  };
  // rows of accumulator register group g (4 registers) of row tile i: wp*WTP + i*32 + 8*g + 4*(lane/32) + 0..3
  auto row_of = [&](int i, int g) { return wp * WTP + i * 32 + 8 * g + 4 * (lane >> 5); };

  // The scale factors of a whole row tile (its four register groups).  The phase ends and the
  // epilogue walk the row tiles and ask for the factors of row tile i + 1 before they work on row
  // tile i: asked for group by group, every group paid a memory round trip of its own with nothing
  // to do meanwhile (16 per phase end; in per-head mode, with 16 phase ends per tile, a fifth of
  // the launch).
  struct RowScales {
    f32x4 rp[4], fp[4];
  };
  auto row_scales = [&](int i, int head, RowScales& r) {
#pragma unroll
    for (int g = 0; g < 4; ++g) pool_scales(row_of(i, g), head, r.rp[g], r.fp[g]);
  };
  // walk the row tiles with the factors of the next one in flight: body(i, factors of row tile i)
  auto for_row_tiles = [&](int head, auto&& body) __attribute__((always_inline)) {
    RowScales cur, nxt;
    row_scales(0, head, cur);
#pragma unroll
    for (int i = 0; i < TP; ++i) {
      if (i + 1 < TP) row_scales(i + 1, head, nxt);
      __builtin_amdgcn_sched_barrier(0);
      body(i, cur);
      __builtin_amdgcn_sched_barrier(0);
      cur = nxt;
    }
  };

  // acc <- acc * (rq * rp)   (end of a K phase)
  auto rescale = [&](int head) {
    float rq[TQ], fq[TQ];
    query_scales(head, rq, fq);
    for_row_tiles(head, [&](int i, const RowScales& rs) __attribute__((always_inline)) {
#pragma unroll
      for (int g = 0; g < 4; ++g)
#pragma unroll
        for (int j = 0; j < TQ; ++j)
#pragma unroll
          for (int e = 0; e < 4; ++e) acc[i][j][4 * g + e] *= rq[j] * rs.rp[g][e];
    });
  };

  // per-head mode: running minimum over heads of the finished head score; acc restarts at 0.
  // A second fp32 register tile does not fit next to a 256x256 accumulator tile, so the running
  // minimum is kept as 16-bit fixed point (score * 32767 rounded to nearest, two per register,
  // packed min): resolution 3.1e-5, error at most 1.6e-5 on a score in [-1, 1].
  constexpr int SM = (MODE == 1) ? 1 : 0;
  int smin[SM ? TP : 1][SM ? TQ : 1][8];
  if (MODE == 1) {
#pragma unroll
    for (int i = 0; i < TP; ++i)
#pragma unroll
      for (int j = 0; j < TQ; ++j)
#pragma unroll
        for (int r = 0; r < 8; ++r) smin[SM ? i : 0][SM ? j : 0][r] = 0x7fff7fff;
  }
  auto finish_head = [&](int head) {
    float rq[TQ], fq[TQ];
    query_scales(head, rq, fq);
    for_row_tiles(head, [&](int i, const RowScales& rs) __attribute__((always_inline)) {
#pragma unroll
      for (int g = 0; g < 4; ++g)
#pragma unroll
        for (int j = 0; j < TQ; ++j)
#pragma unroll
          for (int e = 0; e < 4; e += 2) {
            const float s0 = acc[i][j][4 * g + e] * (fq[j] * rs.fp[g][e]), s1 = acc[i][j][4 * g + e + 1] * (fq[j] * rs.fp[g][e + 1]);
            // the hardware's conversion to signed normalised 16 bit: clamp to [-1, 1], times 32767, round to nearest
            const i16x2 nw = quantise_pair(s0, s1);
            int& slot = smin[SM ? i : 0][SM ? j : 0][2 * g + (e >> 1)];
            slot = __builtin_bit_cast(int, __builtin_elementwise_min(__builtin_bit_cast(i16x2, slot), nw));
            acc[i][j][4 * g + e] = 0.f;
            acc[i][j][4 * g + e + 1] = 0.f;
          }
    });
  };

  // layer-mean mode: when a phase (the K or the V tensor of one layer) ends, the accumulators hold
  // the dot products; |x-y| = sqrt(|x|^2 + |y|^2 - 2 x.y) from the cached squared norms is added
  // to the tile's running sum and the accumulators restart at 0.  Rounding can push the radicand
  // of a near-duplicate pair slightly below 0: it is clamped.  The running sum has no room in the
  // register file next to a 256x256 accumulator tile, so it lives in this workgroup's own 256 KB
  // of the sums buffer (read-modify-write by the lane that owns the element, 0.5 MB per phase
  // against 16 MB of operands); the first phase of a group only writes.  The tile is stored in
  // register order, not row-major: the four values a lane holds for (row tile i, register group
  // g, column tile j) are one 16-byte word at index ((wave*TP + i)*4 + g)*TQ + j)*64 + lane, so
  // every access of a wave is 1 KB contiguous (sum_index() below is the inverse map).
  auto fold = [&](const __amdgpu_buffer_rsrc_t& nQ, const __amdgpu_buffer_rsrc_t& nP, auto first_tag) {
    constexpr bool first = decltype(first_tag)::value;
    typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
    long long tile_lin = ((long long)lz * p.npt + pt) * p.nqt + qt;
    asm volatile("" : "+s"(tile_lin));  // opaque: the addresses are formed here, not kept across the layers
    f32x4* sums = reinterpret_cast<f32x4*>(p.dpart) + tile_lin * (BP * BQ / 4) + (long long)wave * (TP * 4 * TQ * 64) + lane;
    float nq[TQ];
#pragma unroll
    for (int j = 0; j < TQ; ++j)
      nq[j] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(nQ, (q0 + wq * WTQ + j * 32 + (lane & 31)) * 4, 0, 0));
    // one row tile (64 elements of the lane) at a time: all its loads are issued before the first
    // store, so the lane pays one memory round trip per row tile and not one per element
#pragma unroll
    for (int i = 0; i < TP; ++i) {
      f32x4 old[4][TQ];
      f32x4 np[4];
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        np[g] = __builtin_bit_cast(f32x4, (u32x4_t)__builtin_amdgcn_raw_buffer_load_b128(nP, (p0 + row_of(i, g)) * 4, 0, 0));
        if (!first) {
#pragma unroll
          for (int j = 0; j < TQ; ++j) old[g][j] = sums[((i * 4 + g) * TQ + j) * 64];
        }
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int g = 0; g < 4; ++g)
#pragma unroll
        for (int j = 0; j < TQ; ++j) {
          f32x4 d;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float d2 = fmaf(-2.f, acc[i][j][4 * g + e], nq[j] + np[g][e]);
            d[e] = __builtin_amdgcn_sqrtf(fmaxf(d2, 0.f));
            if (!first) d[e] += old[g][j][e];
            acc[i][j][4 * g + e] = 0.f;
          }
          sums[((i * 4 + g) * TQ + j) * 64] = d;
        }
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  // ---- main loop.  Per step: wait for this step's slices, barrier, then compute while refilling
  // the stages the barrier has just freed (query slice of the next step, pool slice of the step
  // after).  The query loads are issued before the pool loads, so "at most LA loads outstanding"
  // means exactly: everything but the newest pool slice has landed.
  // prologue: query slice 0, pool slices 0 and 1.  It leaves the query feed prepared for slice 1 (the
  // loads of step 0) and the pool feed on slice 1: the slots of step 0 move it on to slice 2.
  auto prologue = [&]() {
    prepare(fb, srdBk, srdBv, ringB, B_STAGE);
#pragma unroll
    for (int i = 0; i < LB; ++i) dmaB(i);
    next(fb, SB);
    prepare(fb, srdBk, srdBv, ringB, B_STAGE);
    prepare(fa, srdAk, srdAv, ringA, A_STAGE);
#pragma unroll
    for (int i = 0; i < LA; ++i) dmaA(i);
    next(fa, SA);
    prepare(fa, srdAk, srdAv, ringA, A_STAGE);
#pragma unroll
    for (int i = 0; i < LA; ++i) dmaA(i);
    rdA = rdB = 0;
    sA_next = s_ring;
    sB_next = s_ring + SA * A_STAGE;
  };
  prologue();
  auto step = [&](auto fast_tag) __attribute__((always_inline)) {
    const char *sA = sA_next, *sB = sB_next;
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(LA) : "memory");  // all but the newest pool slice landed
    __syncthreads();  // ... for every wave, and the stages read in the previous step are free
    compute(fast_tag, sA, sB);
  };
  auto run_phase = [&]() __attribute__((always_inline)) {
    clear_pending();
    // the accumulators enter the loops in their accumulation registers: without this the code of the
    // phase end before (the rescale and its loads) is scheduled into the first loop, waits included
#pragma unroll
    for (int i = 0; i < TP; ++i)
#pragma unroll
      for (int j = 0; j < TQ; ++j) asm volatile("" : "+a"(acc[i][j]));
    int u = 0;
    // step u loads pool slice u + 2 and query slice u + 1 of the phase: inside the phase up to u = sps - 3
    for (; u + 2 < sps; ++u) step(std::true_type{});
    for (; u < sps; ++u) step(std::false_type{});
    drain();
  };
  if (MODE == 0) {
    run_phase();
    rescale(0);
    run_phase();
  } else if (MODE == 1) {
    for (int h = 0; h < p.H; ++h) {
      run_phase();
      rescale(h);
      run_phase();
      finish_head(h);
    }
  } else if (MODE == 3) {
    run_phase();
  } else if (MODE == 4) {
    run_phase();
    rescale(split);
    run_phase();
  } else {
    for (int li = 0;;) {
      run_phase();
      if (li == 0)
        fold(nQk, nPk, std::true_type{});
      else
        fold(nQk, nPk, std::false_type{});
      run_phase();
      fold(nQv, nPv, std::false_type{});
      if (++li == nl) break;
      // next layer of the group: the pipeline restarts from an empty ring
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __syncthreads();  // every wave has read its last fragments and its surplus refills have landed
      l = l_first + li;
      set_layer_tensors();
      set_layer_norms();
      fa = Feed{{0, 0}, 0, srdAk, 0, 0};
      fb = Feed{{0, 0}, 0, srdBk, 0, 0};
      prologue();
    }
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the surplus refills of the last steps have landed
  claim_next();

  if (MODE == 2) continue;  // the sums of this group's layers are in place, tile by tile in register order

  if (SHARES) {
    // this share of the tile's scores (MODE 4: the score of head `split`), in register order like
    // the sums of the layer-mean mode: shares are laid out [layer][share][pool tile][query tile]
    const int head = (MODE == 4) ? split : 0;
    float rq[TQ], fq[TQ];
    query_scales(head, rq, fq);
    const long long tile_lin = (((long long)lz * p.S + split) * p.npt + pt) * p.nqt + qt;
    f32x4* out = reinterpret_cast<f32x4*>(p.dpart) + tile_lin * (BP * BQ / 4) + (long long)wave * (TP * 4 * TQ * 64) + lane;
    for_row_tiles(head, [&](int i, const RowScales& rs) __attribute__((always_inline)) {
#pragma unroll
      for (int g = 0; g < 4; ++g)
#pragma unroll
        for (int j = 0; j < TQ; ++j) {
          f32x4 d;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            // fq fp = aVq aVp / 2; rq rp = (aKq aKp) / (aVq aVp); in MODE 4 the K part was rescaled at the phase end
            const float f = (MODE == 3 && p.raw)      ? 1.f
                            : (MODE == 4 || split_v) ? fq[j] * rs.fp[g][e]
                                                     : (rq[j] * fq[j]) * (rs.rp[g][e] * rs.fp[g][e]);
            d[e] = acc[i][j][4 * g + e] * f;
          }
          out[((i * 4 + g) * TQ + j) * 64] = d;
        }
    });
    continue;
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
    float rq[TQ], fq[TQ];
    if (MODE == 0) query_scales(0, rq, fq);
    // dead blocks and rows past the end of the pool: -inf.  The flags of row tile i + 1 are asked for
    // with its scale factors, before the work on row tile i.
    struct RowBias {
      f32x4 b[4];
    };
    auto row_bias = [&](int i, RowBias& r) {
#pragma unroll
      for (int g = 0; g < 4; ++g)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int gp = p0 + row_of(i, g) + e;
          r.b[g][e] = (gp < p.P && (!p.live || p.live[(long long)l * p.P + gp])) ? 0.f : -INFINITY;
        }
    };
    RowScales cur, nxt;
    RowBias bcur, bnxt;
    if (MODE == 0) row_scales(0, 0, cur);
    row_bias(0, bcur);
#pragma unroll
    for (int i = 0; i < TP; ++i) {
      if (i + 1 < TP) {
        if (MODE == 0) row_scales(i + 1, 0, nxt);
        row_bias(i + 1, bnxt);
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int row = row_of(i, g);
#pragma unroll
        for (int j = 0; j < TQ; ++j)
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            float sc;
            if (MODE == 0)
              sc = acc[i][j][4 * g + e] * (fq[j] * cur.fp[g][e]) + bcur.b[g][e];
            else
              sc = (float)__builtin_bit_cast(i16x2, smin[SM ? i : 0][SM ? j : 0][2 * g + (e >> 1)])[e & 1] / 32767.f + bcur.b[g][e];
            top2_push(sc, p0 + row + e, best[j], bidx[j], second[j]);
          }
      }
      __builtin_amdgcn_sched_barrier(0);
      cur = nxt;
      bcur = bnxt;
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
  __syncthreads();  // every wave is done reading the ring: its first bytes become the merge scratch
  Part* s_part = reinterpret_cast<Part*>(s_ring);  // [WP][BQ]
  if (lane < 32) {
#pragma unroll
    for (int j = 0; j < TQ; ++j) {
      Part t;
      t.best = best[j];
      t.idx = bidx[j];
      t.second = second[j];
      t.pad = 0;
      s_part[wp * BQ + wq * WTQ + j * 32 + lane] = t;
    }
  }
  __syncthreads();
  if (tid < BQ && q0 + tid < p.Q) {
    Part t = s_part[tid];
#pragma unroll
    for (int w = 1; w < WP; ++w) {
      const Part u = s_part[w * BQ + tid];
      top2_merge(t.best, t.idx, t.second, u.best, u.idx, u.second);
    }
    p.part[((long long)l * p.npt + pt) * p.Q + q0 + tid] = t;
  }
  }  // next tile of this workgroup
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

// Float index of element (row r, column c) of a 256x256 tile of sums as the tile kernel stores it
// (2x2 waves of 128x128, four 32-row tiles x four 32-column tiles per wave, register group g holds
// rows 8g + 4*(lane/32) + 0..3 of a row tile): r is a multiple of 4, the four rows r..r+3 follow.
__device__ __forceinline__ int sum_index(int r, int c) {
  const int wave = (r >> 7) * 2 + (c >> 7);
  const int i = (r >> 5) & 3, g = (r >> 3) & 3, half = (r >> 2) & 1, j = (c >> 5) & 3;
  const int lane = half * 32 + (c & 31);
  return ((((wave * 4 + i) * 4 + g) * 4 + j) * 64 + lane) * 4;
}

// Selection from tiles of sums (one 256x256 tile after the other per group, each in the tile
// kernel's register order): the value of a pair is -scale times the sum of its element over the
// groups.  Layer-mean mode: groups = groups of layers, scale = 1/(2dhN), so "higher wins, equal
// goes to the lower index" on -distance picks the nearest live pool block.  Split mode: groups =
// the shares of a tile's reduction, scale = -1, the value is the score; blockIdx.z is the layer.
// take_min: the groups are combined by the minimum instead of the sum (per-head-all score, one
// share per head).
// grid = (query tiles of 64, pool chunks of sel_rows rows, layers); sel_rows is a multiple of 16;
// a thread owns one query column and every fourth group of four rows.
__global__ __launch_bounds__(256) void tile_sums_select_kernel(const float* __restrict__ dpart, int groups, int P,
                                                               int Q, int npt, int nqt, int sel_rows, float scale,
                                                               int take_min, const uint8_t* __restrict__ live,
                                                               Part* __restrict__ part) {
  __shared__ Part s_part[4][64];
  const int tq = threadIdx.x & 63, tp = threadIdx.x >> 6;
  const int q = blockIdx.x * 64 + tq;
  const int pbeg = blockIdx.y * sel_rows, pend = min(P, pbeg + sel_rows);
  const long long gstride = (long long)npt * nqt * 65536;
  dpart += (long long)blockIdx.z * groups * gstride;
  if (live) live += (long long)blockIdx.z * P;
  part += (long long)blockIdx.z * gridDim.y * Q;
  float best = -INFINITY, second = -INFINITY;
  int bidx = -1;
  if (q < Q) {
    for (int r = pbeg + 4 * tp; r < pend; r += 16) {
      const float* src = dpart + ((long long)(r >> 8) * nqt + (q >> 8)) * 65536 + sum_index(r & 255, q & 255);
      f32x4 sum = {0.f, 0.f, 0.f, 0.f};  // groups are added in ascending order: the same bits on every run
      if (take_min) {
        // per-head-all score: every head's score goes onto the grid of 1/32767 first, exactly as the
        // whole-tile path keeps its running minimum, so that a pair reports the same bits on both paths
        int qmin[4] = {32767, 32767, 32767, 32767};
        for (int g = 0; g < groups; ++g) {
          const f32x4 v = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(src + g * gstride));
#pragma unroll
          for (int e = 0; e < 4; e += 2) {
            const i16x2 q = quantise_pair(v[e], v[e + 1]);
            qmin[e] = min(qmin[e], (int)q[0]);
            qmin[e + 1] = min(qmin[e + 1], (int)q[1]);
          }
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) sum[e] = (float)qmin[e] / 32767.f;
      } else {
        int g = 0;
        for (; g + 4 <= groups; g += 4) {
          f32x4 v[4];
#pragma unroll
          for (int u = 0; u < 4; ++u) v[u] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(src + (g + u) * gstride));
#pragma unroll
          for (int u = 0; u < 4; ++u) sum += v[u];
        }
        for (; g < groups; ++g) sum += __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(src + g * gstride));
      }
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (r + e < pend && (!live || live[r + e])) top2_push(-(sum[e] * scale), r + e, best, bidx, second);
    }
  }
  Part t;
  t.best = best;
  t.idx = bidx;
  t.second = second;
  t.pad = 0;
  s_part[tp][tq] = t;
  __syncthreads();
  if (tp == 0 && q < Q) {
#pragma unroll
    for (int w = 1; w < 4; ++w) {
      const Part u = s_part[w][tq];
      top2_merge(t.best, t.idx, t.second, u.best, u.idx, u.second);
    }
    part[(long long)blockIdx.y * Q + q] = t;
  }
}

// Layer-mean distance from the shares of a split reduction (few tiles: every tile's reduction was cut into
// `shares` workgroups, the first half on the K tensor, the second on V, each storing its bare partial dot
// products as a tile in register order, laid out [layer][share][pool tile][query tile]).  Per pair and layer the
// shares of each tensor are added in ascending order, |x - y| = sqrt(max(|x|^2 + |y|^2 - 2 x.y, 0)) is formed
// from the cached squared norms exactly as the whole-tile path folds it, the layers are added in ascending
// order, and the selection is the one of tile_sums_select_kernel (top-2 on -distance, dead and tail rows out).
__global__ __launch_bounds__(256) void layer_mean_shares_select_kernel(
    const float* __restrict__ dpart, int shares, int L, int P, int Q, int npt, int nqt, int sel_rows, float scale,
    const uint8_t* __restrict__ live, const float* __restrict__ q_ksq, const float* __restrict__ q_vsq,
    const float* __restrict__ p_ksq, const float* __restrict__ p_vsq, Part* __restrict__ part) {
  __shared__ Part s_part[4][64];
  const int tq = threadIdx.x & 63, tp = threadIdx.x >> 6;
  const int q = blockIdx.x * 64 + tq;
  const int pbeg = blockIdx.y * sel_rows, pend = min(P, pbeg + sel_rows);
  const long long gstride = (long long)npt * nqt * 65536;
  float best = -INFINITY, second = -INFINITY;
  int bidx = -1;
  if (q < Q) {
    for (int r = pbeg + 4 * tp; r < pend; r += 16) {
      const float* src = dpart + ((long long)(r >> 8) * nqt + (q >> 8)) * 65536 + sum_index(r & 255, q & 255);
      f32x4 dist = {0.f, 0.f, 0.f, 0.f};
      for (int l = 0; l < L; ++l) {
        const float* lsrc = src + (long long)l * shares * gstride;
        f32x4 dot[2];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          dot[t] = f32x4{0.f, 0.f, 0.f, 0.f};
          for (int g = 0; g < shares / 2; ++g)
            dot[t] += __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(lsrc + (long long)(t * (shares / 2) + g) * gstride));
        }
        const float nqk = q_ksq[(long long)l * Q + q], nqv = q_vsq[(long long)l * Q + q];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          if (r + e >= pend) continue;
          const float npk = p_ksq[(long long)l * P + r + e], npv = p_vsq[(long long)l * P + r + e];
          dist[e] += __builtin_amdgcn_sqrtf(fmaxf(fmaf(-2.f, dot[0][e], nqk + npk), 0.f));
          dist[e] += __builtin_amdgcn_sqrtf(fmaxf(fmaf(-2.f, dot[1][e], nqv + npv), 0.f));
        }
      }
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (r + e < pend && (!live || live[r + e])) top2_push(-(dist[e] * scale), r + e, best, bidx, second);
    }
  }
  Part t;
  t.best = best;
  t.idx = bidx;
  t.second = second;
  t.pad = 0;
  s_part[tp][tq] = t;
  __syncthreads();
  if (tp == 0 && q < Q) {
#pragma unroll
    for (int w = 1; w < 4; ++w) {
      const Part u = s_part[w][tq];
      top2_merge(t.best, t.idx, t.second, u.best, u.idx, u.second);
    }
    part[(long long)blockIdx.y * Q + q] = t;
  }
}

// rows of the pool per selection workgroup: about 2048 workgroups, at least 32 rows each
inline int select_rows(int64_t P, int64_t Q) {
  const int64_t qtiles = (Q + 63) / 64;
  int64_t chunks = 2048 / (qtiles > 0 ? qtiles : 1);
  if (chunks < 1) chunks = 1;
  int64_t rows = (P + chunks - 1) / chunks;
  rows = (rows + 31) / 32 * 32;
  return (int)(rows < 32 ? 32 : rows);
}

// 64 queries per workgroup, four threads per query, each merging every fourth chunk.
__global__ __launch_bounds__(256) void layer_mean_finalize_kernel(const Part* __restrict__ part, int nchunks, int Q,
                                                                  float thr, int32_t* __restrict__ best_idx,
                                                                  float* __restrict__ best_dist,
                                                                  int32_t* __restrict__ match_idx,
                                                                  float* __restrict__ second_dist) {
  __shared__ Part s_part[4][64];
  const int tq = threadIdx.x & 63, tc = threadIdx.x >> 6;
  const int q = blockIdx.x * 64 + tq;
  Part t;
  t.best = -INFINITY;
  t.second = -INFINITY;
  t.idx = -1;
  t.pad = 0;
  if (q < Q)
    for (int c = tc; c < nchunks; c += 4) {
      const Part u = part[(long long)c * Q + q];
      top2_merge(t.best, t.idx, t.second, u.best, u.idx, u.second);
    }
  s_part[tc][tq] = t;
  __syncthreads();
  if (tc != 0 || q >= Q) return;
#pragma unroll
  for (int w = 1; w < 4; ++w) {
    const Part u = s_part[w][tq];
    top2_merge(t.best, t.idx, t.second, u.best, u.idx, u.second);
  }
  best_idx[q] = t.idx;
  best_dist[q] = -t.best;
  match_idx[q] = (t.idx >= 0 && -t.best <= thr) ? t.idx : -1;
  if (second_dist) second_dist[q] = -t.second;
}

// Layer-mean mode: how the L layers are split into groups.  A workgroup walks the layers of one
// group, so large problems (many tiles) use one group and write every sum once; small ones split
// the layers until there are enough workgroups to fill the chip.
struct LayerSplit {
  int G, groups;
};
inline LayerSplit layer_split(int L, int64_t tiles) {
  int64_t want = (1024 + tiles - 1) / (tiles > 0 ? tiles : 1);
  if (want < 1) want = 1;
  if (want > L) want = L;
  LayerSplit r;
  r.G = (int)((L + want - 1) / want);
  r.groups = (L + r.G - 1) / r.G;
  return r;
}

// Compute units of the current device (a workgroup of the tile kernel fills one): the size of the
// first round of workgroups.
inline int compute_units() {
  static thread_local int cached_dev = -1, cached_cus = 0;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 0;
  if (dev != cached_dev) {
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) cus = 0;
    cached_dev = dev;
    cached_cus = cus;
  }
  return cached_cus;
}
// Workgroups of a tile-kernel launch: one per compute unit (the kernel's 160 KB of LDS allow no more), a multiple
// of the 8 XCDs so that a workgroup's virtual indices keep their XCD; never more than there are virtual workgroups.
inline unsigned launch_grid(unsigned vgrid) {
  int cus = compute_units() / 8 * 8;
  if (cus > kMaxGrid) cus = kMaxGrid;
  return (cus > 0 && (unsigned)cus < vgrid) ? (unsigned)cus : vgrid;
}
// What a launch of more than one round keeps behind the rest of the workspace: the header (counters and progress
// words, 128 bytes each) and one claim word per slot of every workgroup's walk.
constexpr int kChunk = 32;
constexpr int kStealMin = 64;
constexpr int kTailShare = 10;   // the last tenth of every list can be taken from its back
constexpr int kDynamicRounds = 16;  // launches of fewer rounds keep the fixed schedule: nothing to gain there
inline int64_t virtual_grid(int64_t total) { return (total + 8 * kChunk - 1) / (8 * kChunk) * (8 * kChunk); }
inline size_t schedule_bytes(int64_t total) {
  // the walks of a launch with fewer workgroups than kMaxGrid are longer; together they never hold more than
  // one slot per virtual workgroup plus one per workgroup
  return (size_t)(kScheduleHeader + virtual_grid(total > 0 ? total : 1) + kMaxGrid) * sizeof(int);
}
__global__ void clear_schedule_kernel(int* ctr, int n) {
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) ctr[i] = 0;
}
// Sets mp.ctr for a launch of `grid` workgroups over mp.vgrid virtual ones: counters and claims (cleared on the
// stream) when the launch has many rounds, a fixed schedule otherwise.  Measured on two shapes of 64 and 192
// rounds: 2 to 3 % less time than the fixed schedule with the last tenth of the lists open to the other XCDs'
// workgroups; with every slot claimed, 4 % MORE than the fixed schedule (a swap per tile costs that much).
inline rc_status prepare_schedule(MatchParams& mp, unsigned grid, void* schedule, hipStream_t st) {
  mp.ctr = nullptr;
  mp.rounds = 0;
  mp.steal_min = kStealMin;
  mp.dyn_from = 0;
  if ((unsigned)mp.vgrid < kDynamicRounds * grid || !schedule) return RC_OK;
  mp.ctr = static_cast<int*>(schedule);
  const int per_list = (int)grid / 8;
  mp.rounds = (mp.vgrid / 8 + per_list - 1) / per_list;
  mp.dyn_from = mp.vgrid / 8 - (mp.vgrid / 8) / kTailShare;
  const int n = kScheduleHeader + (int)grid * mp.rounds;
  clear_schedule_kernel<<<(n + 1023) / 1024 < 64 ? (n + 1023) / 1024 : 64, 1024, 0, st>>>(mp.ctr, n);
  return check_launch("rc_match_blocks(tile schedule)");
}
constexpr int kStaggerUnit = 6;  // x 1024 clocks per tile index, one to two pipeline steps (flat optimum between 3 and 8)

// Tile shape: a 128x128 accumulator tile per wave (all 256 accumulation registers of a lane) in
// every mode.  What is carried across phases is kept out of the fp32 register budget: the
// per-head mode packs its running minimum into 16-bit fixed point, the layer-mean mode keeps
// its running sum in the workspace.
struct TileShape {
  int bp, bq;
};
constexpr TileShape kBlockTile = {256, 256};
constexpr TileShape kHeadTile = {256, 256};
// Few query blocks (a decoding step of a handful of requests): a 64-column tile does a quarter of
// the matrix work per pool slice and leaves the kernel to the speed of the pool stream.
constexpr TileShape kNarrowTile = {256, 64};
constexpr TileShape kMidTile = {256, 128};

inline TileShape tile_for(int mode, int64_t Q) {
  if (mode != RC_SCORE_BLOCK) return kHeadTile;
  return Q <= kNarrowTile.bq ? kNarrowTile : Q <= kMidTile.bq ? kMidTile : kBlockTile;
}

// byte offset of the selection partials inside the layer-mean workspace (after the sums: one
// 256x256 tile of floats per (group, pool tile, query tile))
inline size_t layer_mean_part_offset(int groups, int64_t npt, int64_t nqt) {
  return (size_t)groups * (size_t)npt * (size_t)nqt * 65536 * sizeof(float);
}

// A tile kernel launch runs in rounds of one workgroup per compute unit, and a problem with few
// tiles (a call for one layer, a small pool) leaves most of the chip idle or pays a whole round
// for a few left-over tiles.  Such problems split the reduction of every tile over S workgroups
// (S even: half of them on the K tensor, half on V).  S is the power of two with the lowest
// estimated time, in units of one pipeline step:
//   rounds(S) * (steps of a share + 6 for filling the pipeline and storing the share)
//   + 0.03 per tile share for the pass that adds the shares + 5 for its launch,
// and the split is used when that is at least 10 % below the estimate for whole tiles.  The
// constants come from measurements of 1 to 144 tiles of the 256 x 256 shape (within 10 % from 64
// tiles up; a single layer of 16 tiles takes 143 us against 112 estimated).  A share has at least
// 8 steps; the shares of all tiles take at most 512 MB; problems of more than one round are left
// alone.  In per-head mode the shares are the H heads (the score is a minimum over heads, not a
// sum over the reduction), chosen by the same estimate.  With at most 128 query blocks the whole-tile
// path has its narrow tiles, so the split is only used below half a round there.  Block mode only.
// The decision depends on the shape alone (an MI355X has 256 compute units), so that the workspace
// size does not depend on the device that happens to be current.
constexpr int kSplitComputeUnits = 256;
inline int split_count(int mode, int64_t L, int64_t P, int64_t Q, int T, int H) {
  if (P <= 0 || Q <= 0 || L <= 0) return 1;
  const int64_t tiles = L * ((P + 255) / 256) * ((Q + 255) / 256);
  if (tiles > kSplitComputeUnits) return 1;  // more than one round: measured gains of 0-6 % only (workgroups of
                                             // later rounds start as earlier ones end, the rounds are not that rigid)
  if (mode == RC_SCORE_PER_HEAD_ALL) {
    if (H < 2 || tiles * H > 2048) return 1;
    auto rounds = [&](int64_t wgs) { return (double)((wgs + kSplitComputeUnits - 1) / kSplitComputeUnits); };
    const double whole = rounds(tiles) * (4.0 * T * H + 6.0);
    const double heads = rounds(tiles * H) * (4.0 * T + 6.0) + 0.03 * (double)(tiles * H) + 5.0;
    return heads < 0.9 * whole ? H : 1;
  }
  if (Q <= 128 && tiles * 2 > kSplitComputeUnits) return 1;
  const int steps = T * H * 128 / kBK;  // per tensor
  auto estimate = [&](int S) {
    const double rounds = (double)((tiles * S + kSplitComputeUnits - 1) / kSplitComputeUnits);
    return rounds * (2.0 * steps / S + 6.0) + (S > 1 ? 0.03 * (double)(tiles * S) + 5.0 : 0.0);
  };
  int best = 1;
  double best_cost = 0.9 * estimate(1);
  for (int S = 2; tiles * S <= 2048 && 2 * steps / S >= 8 && steps % (S / 2) == 0; S *= 2) {
    const double c = estimate(S);
    if (c < best_cost) {
      best_cost = c;
      best = S;
    }
  }
  return best;
}

struct SplitLayout {
  int S;
  int64_t npt, nqt;
  int sel_rows;
  int64_t nchunks;
  size_t part_offset, bytes;
};
inline SplitLayout split_layout(int S, int64_t L, int64_t P, int64_t Q) {
  SplitLayout r;
  r.S = S;
  r.npt = (P + 255) / 256;
  r.nqt = (Q + 255) / 256;
  r.sel_rows = select_rows(P, Q);
  r.nchunks = (P + r.sel_rows - 1) / r.sel_rows;
  r.part_offset = (size_t)L * (size_t)S * (size_t)r.npt * (size_t)r.nqt * 65536 * sizeof(float);
  r.bytes = r.part_offset + (size_t)L * (size_t)r.nchunks * (size_t)Q * sizeof(Part);
  return r;
}

template <bool BF16>
void launch_tiles(int mode, const MatchParams& mp, unsigned grid, hipStream_t st) {
  if (mode == RC_SCORE_BLOCK && mp.Q <= kNarrowTile.bq)
    match_tile_kernel<BF16, kNarrowTile.bp, kNarrowTile.bq, 0><<<grid, kThreads, 0, st>>>(mp);
  else if (mode == RC_SCORE_BLOCK && mp.Q <= kMidTile.bq)
    match_tile_kernel<BF16, kMidTile.bp, kMidTile.bq, 0><<<grid, kThreads, 0, st>>>(mp);
  else if (mode == RC_SCORE_BLOCK && mp.nqt > 1)
    match_tile_kernel<BF16, kBlockTile.bp, kBlockTile.bq, 0, true><<<grid, kThreads, 0, st>>>(mp);
  else if (mode == RC_SCORE_BLOCK)
    match_tile_kernel<BF16, kBlockTile.bp, kBlockTile.bq, 0><<<grid, kThreads, 0, st>>>(mp);
  else
    match_tile_kernel<BF16, kHeadTile.bp, kHeadTile.bq, 1><<<grid, kThreads, 0, st>>>(mp);
}

}  // namespace
}  // namespace rc

extern "C" size_t rc_match_workspace_size(const rc_kv_desc* qdesc, int32_t mode, int64_t Q, int64_t P) {
  using namespace rc;
  if (!qdesc || Q < 0 || P < 0 || qdesc->n_layers < 0) return 0;
  if (mode != RC_SCORE_BLOCK && mode != RC_SCORE_PER_HEAD_ALL) return 0;
  const int S = split_count(mode, qdesc->n_layers, P, Q, qdesc->block_tokens, qdesc->n_kv_heads);
  if (S > 1) return split_layout(S, qdesc->n_layers, P, Q).bytes;
  const TileShape ts = tile_for(mode, Q);
  const int64_t npt = (P + ts.bp - 1) / ts.bp;
  const int64_t nqt = (Q + ts.bq - 1) / ts.bq;
  const int64_t n = (int64_t)qdesc->n_layers * (npt > 0 ? npt : 1) * Q;
  return (size_t)(n > 0 ? n : 1) * sizeof(Part) + schedule_bytes((int64_t)qdesc->n_layers * npt * nqt);
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
  const TileShape ts = tile_for(mode, Q);
  const int64_t npt = (P + ts.bp - 1) / ts.bp, nqt = (Q + ts.bq - 1) / ts.bq;
  const int64_t total = (int64_t)L * npt * nqt;
  if (Q > 0x7fffffffLL || P > 0x7fffffffLL || total > 0x3fffffffLL || (int64_t)L * Q > 0x7fffffffLL * 128)
    return fail(RC_ERR_UNSUPPORTED, "rc_match_blocks: problem beyond the grid limits");
  const size_t need = rc_match_workspace_size(qdesc, mode, Q, P);
  if (!workspace || workspace_bytes < need || !aligned16(workspace))
    return fail(RC_ERR_WORKSPACE, "rc_match_blocks: workspace of %zu bytes needed (16-byte aligned), got %zu", need,
                workspace_bytes);
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const int S = split_count(mode, L, P, Q, qdesc->block_tokens, qdesc->n_kv_heads);
  const long long LQ = (long long)L * Q;

  if (S > 1) {
    // few tiles: shares of every tile's reduction, then sum + selection, then the merge over pool chunks
    const SplitLayout sl = split_layout(S, L, P, Q);
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
    mp.part = nullptr;
    mp.dpart = static_cast<float*>(workspace);
    mp.q_lstride_b = qdesc->layer_stride * 2;
    mp.p_lstride_b = pdesc->layer_stride * 2;
    mp.L = L;
    mp.Q = (int)Q;
    mp.P = (int)P;
    mp.T = qdesc->block_tokens;
    mp.H = qdesc->n_kv_heads;
    mp.npt = (int)sl.npt;
    mp.nqt = (int)sl.nqt;
    mp.total = (int)(L * sl.npt * sl.nqt * S);
    mp.chunk = kChunk;
    mp.raw = 0;
    mp.G = 1;
    mp.S = S;
    mp.stagger_wgs = 0;
    mp.stagger_unit = 0;
    mp.vgrid = (int)virtual_grid(mp.total);
    const unsigned grid = launch_grid((unsigned)mp.vgrid);
    mp.ctr = nullptr;
    mp.rounds = 0;
    mp.steal_min = 0;
    mp.dyn_from = 0;
    const bool heads = mode == RC_SCORE_PER_HEAD_ALL;
    if (qdesc->dtype == RC_BF16) {
      if (heads)
        match_tile_kernel<true, 256, 256, 4><<<grid, kThreads, 0, st>>>(mp);
      else
        match_tile_kernel<true, 256, 256, 3><<<grid, kThreads, 0, st>>>(mp);
    } else {
      if (heads)
        match_tile_kernel<false, 256, 256, 4><<<grid, kThreads, 0, st>>>(mp);
      else
        match_tile_kernel<false, 256, 256, 3><<<grid, kThreads, 0, st>>>(mp);
    }
    if (rc_status s = check_launch("rc_match_blocks(tile shares)")) return s;
    Part* part = reinterpret_cast<Part*>(static_cast<char*>(workspace) + sl.part_offset);
    const dim3 sgrid((unsigned)((Q + 63) / 64), (unsigned)sl.nchunks, (unsigned)L);
    tile_sums_select_kernel<<<sgrid, 256, 0, st>>>(mp.dpart, S, (int)P, (int)Q, (int)sl.npt, (int)sl.nqt, sl.sel_rows,
                                                   -1.0f, heads ? 1 : 0, pool_live, part);
    if (rc_status s = check_launch("rc_match_blocks(select)")) return s;
    match_finalize_kernel<<<(unsigned)((LQ + 255) / 256), 256, 0, st>>>(part, (int)sl.nchunks, LQ, (int)Q, tau, best_idx,
                                                                       best_score, match_idx, second_score);
    return check_launch("rc_match_blocks(finalize)");
  }

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
    mp.chunk = kChunk;
    mp.raw = 0;
    mp.dpart = nullptr;
    mp.G = 1;
    mp.S = 1;
    mp.stagger_wgs = compute_units();
    mp.stagger_unit = kStaggerUnit;
    mp.vgrid = (int)virtual_grid(total);
    const unsigned grid = launch_grid((unsigned)mp.vgrid);
    if (rc_status s = prepare_schedule(mp, grid, static_cast<char*>(workspace) + need - schedule_bytes(total), st)) return s;
    if (qdesc->dtype == RC_BF16)
      launch_tiles<true>(mode, mp, grid, st);
    else
      launch_tiles<false>(mode, mp, grid, st);
    if (rc_status s = check_launch("rc_match_blocks(tiles)")) return s;
  }
  match_finalize_kernel<<<(unsigned)((LQ + 255) / 256), 256, 0, st>>>(static_cast<const Part*>(workspace), (int)npt, LQ,
                                                                     (int)Q, tau, best_idx, best_score, match_idx,
                                                                     second_score);
  return check_launch("rc_match_blocks(finalize)");
}

extern "C" size_t rc_layer_mean_workspace_size(const rc_kv_desc* qdesc, int64_t Q, int64_t P) {
  using namespace rc;
  if (!qdesc || Q < 0 || P < 0 || qdesc->n_layers <= 0) return 0;
  const int64_t npt = (P + kBlockTile.bp - 1) / kBlockTile.bp, nqt = (Q + kBlockTile.bq - 1) / kBlockTile.bq;
  const int S = split_count(RC_SCORE_BLOCK, qdesc->n_layers, P, Q, qdesc->block_tokens, qdesc->n_kv_heads);
  if (S > 1) return split_layout(S, qdesc->n_layers, P, Q).bytes;  // few tiles: shares of every tile's reduction
  const LayerSplit ls = layer_split(qdesc->n_layers, npt * nqt);
  const int sel_rows = select_rows(P, Q);
  const int64_t nchunks = (P + sel_rows - 1) / sel_rows;
  return layer_mean_part_offset(ls.groups, npt, nqt) + (size_t)(nchunks > 0 ? nchunks : 1) * (size_t)(Q > 0 ? Q : 1) * sizeof(Part);
}

extern "C" rc_status rc_match_blocks_layer_mean(const rc_kv_desc* qdesc, const rc_kv_desc* pdesc, const void* kq,
                                                const void* vq, int64_t Q, const float* q_ksq, const float* q_vsq,
                                                const void* kp, const void* vp, int64_t P, const float* p_ksq,
                                                const float* p_vsq, const uint8_t* pool_live, float threshold,
                                                int32_t* best_idx, float* best_dist, int32_t* match_idx,
                                                float* second_dist, void* workspace, size_t workspace_bytes,
                                                void* hip_stream) {
  using namespace rc;
  clear_error();
  if (rc_status s = check_desc(qdesc, Q, "rc_match_blocks_layer_mean(query)")) return s;
  if (rc_status s = check_desc(pdesc, P, "rc_match_blocks_layer_mean(pool)")) return s;
  if (qdesc->n_layers != pdesc->n_layers || qdesc->block_tokens != pdesc->block_tokens ||
      qdesc->n_kv_heads != pdesc->n_kv_heads || qdesc->head_dim != pdesc->head_dim || qdesc->dtype != pdesc->dtype)
    return fail(RC_ERR_INVALID_ARG, "rc_match_blocks_layer_mean: query and pool descriptors differ in more than layer_stride");
  if (!(threshold == threshold)) return fail(RC_ERR_INVALID_ARG, "rc_match_blocks_layer_mean: threshold is NaN");
  const int L = qdesc->n_layers;
  if (L <= 0) return fail(RC_ERR_INVALID_ARG, "rc_match_blocks_layer_mean: a mean over %d layers is undefined", L);
  if (Q == 0) return RC_OK;
  if (!kq || !vq || !q_ksq || !q_vsq || !best_idx || !best_dist || !match_idx)
    return fail(RC_ERR_INVALID_ARG, "rc_match_blocks_layer_mean: NULL query or output pointer");
  if (P > 0 && (!kp || !vp || !p_ksq || !p_vsq))
    return fail(RC_ERR_INVALID_ARG, "rc_match_blocks_layer_mean: NULL pool pointer");
  if (!aligned16(kq) || !aligned16(vq) || !aligned16(kp) || !aligned16(vp))
    return fail(RC_ERR_INVALID_ARG, "rc_match_blocks_layer_mean: KV pointer not 16-byte aligned");
  const TileShape ts = kBlockTile;
  const int64_t npt = (P + ts.bp - 1) / ts.bp, nqt = (Q + ts.bq - 1) / ts.bq;
  const LayerSplit ls = layer_split(L, npt * nqt);
  const int64_t total = (int64_t)ls.groups * npt * nqt;
  if (Q > 0x7fffffffLL || P > 0x7fffffffLL || total > 0x3fffffffLL || Q > (1LL << 20))
    return fail(RC_ERR_UNSUPPORTED, "rc_match_blocks_layer_mean: problem beyond the grid limits");
  const size_t need = rc_layer_mean_workspace_size(qdesc, Q, P);
  if (!workspace || workspace_bytes < need || !aligned16(workspace))
    return fail(RC_ERR_WORKSPACE, "rc_match_blocks_layer_mean: workspace of %zu bytes needed (16-byte aligned), got %zu",
                need, workspace_bytes);
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  float* dpart = static_cast<float*>(workspace);
  const float scale = 1.0f / ((float)L * 2.0f * (float)qdesc->block_tokens * (float)qdesc->n_kv_heads);
  const int S = split_count(RC_SCORE_BLOCK, L, P, Q, qdesc->block_tokens, qdesc->n_kv_heads);
  if (S > 1) {
    // Few tiles (a call with one or a few layers, a small pool): the launch would leave compute units idle, and
    // giving every workgroup fewer layers does not help below one layer each.  Every tile's reduction is cut into
    // S shares as in rc_match_blocks (half of them on K, half on V), the shares store bare dot products, and the
    // selection kernel forms the distances from their sums.
    const SplitLayout sl = split_layout(S, L, P, Q);
    MatchParams mp;
    mp.kq = static_cast<const char*>(kq);
    mp.vq = static_cast<const char*>(vq);
    mp.kp = static_cast<const char*>(kp);
    mp.vp = static_cast<const char*>(vp);
    mp.q_ksq = q_ksq;
    mp.q_vsq = q_vsq;
    mp.p_ksq = p_ksq;
    mp.p_vsq = p_vsq;
    mp.live = nullptr;
    mp.part = nullptr;
    mp.dpart = dpart;
    mp.q_lstride_b = qdesc->layer_stride * 2;
    mp.p_lstride_b = pdesc->layer_stride * 2;
    mp.L = L;
    mp.Q = (int)Q;
    mp.P = (int)P;
    mp.T = qdesc->block_tokens;
    mp.H = qdesc->n_kv_heads;
    mp.npt = (int)sl.npt;
    mp.nqt = (int)sl.nqt;
    mp.total = (int)(L * sl.npt * sl.nqt * S);
    mp.chunk = kChunk;
    mp.raw = 1;
    mp.G = 1;
    mp.S = S;
    mp.stagger_wgs = 0;
    mp.stagger_unit = 0;
    mp.vgrid = (int)virtual_grid(mp.total);
    const unsigned grid = launch_grid((unsigned)mp.vgrid);
    mp.ctr = nullptr;
    mp.rounds = 0;
    mp.steal_min = 0;
    mp.dyn_from = 0;
    if (qdesc->dtype == RC_BF16)
      match_tile_kernel<true, 256, 256, 3><<<grid, kThreads, 0, st>>>(mp);
    else
      match_tile_kernel<false, 256, 256, 3><<<grid, kThreads, 0, st>>>(mp);
    if (rc_status s = check_launch("rc_match_blocks_layer_mean(tile shares)")) return s;
    Part* part = reinterpret_cast<Part*>(static_cast<char*>(workspace) + sl.part_offset);
    const dim3 sgrid((unsigned)((Q + 63) / 64), (unsigned)sl.nchunks);
    layer_mean_shares_select_kernel<<<sgrid, 256, 0, st>>>(dpart, S, L, (int)P, (int)Q, (int)sl.npt, (int)sl.nqt, sl.sel_rows,
                                                           scale, pool_live, q_ksq, q_vsq, p_ksq, p_vsq, part);
    if (rc_status s = check_launch("rc_match_blocks_layer_mean(select)")) return s;
    layer_mean_finalize_kernel<<<(unsigned)((Q + 63) / 64), 256, 0, st>>>(part, (int)sl.nchunks, (int)Q, threshold, best_idx,
                                                                          best_dist, match_idx, second_dist);
    return check_launch("rc_match_blocks_layer_mean(finalize)");
  }
  Part* part = reinterpret_cast<Part*>(static_cast<char*>(workspace) + layer_mean_part_offset(ls.groups, npt, nqt));
  const int sel_rows = select_rows(P, Q);
  const int64_t nchunks = (P + sel_rows - 1) / sel_rows;
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
    mp.live = nullptr;  // eligibility is applied by the selection kernel
    mp.part = nullptr;
    mp.dpart = dpart;
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
    mp.chunk = kChunk;
    mp.raw = 0;
    mp.G = ls.G;
    mp.S = 1;
    mp.stagger_wgs = compute_units();
    mp.stagger_unit = kStaggerUnit;
    mp.vgrid = (int)virtual_grid(total);
    const unsigned grid = launch_grid((unsigned)mp.vgrid);
    if (rc_status s = prepare_schedule(mp, grid, nullptr, st)) return s;  // a group of layers per tile: few, long tiles
    if (qdesc->dtype == RC_BF16)
      match_tile_kernel<true, kBlockTile.bp, kBlockTile.bq, 2><<<grid, kThreads, 0, st>>>(mp);
    else
      match_tile_kernel<false, kBlockTile.bp, kBlockTile.bq, 2><<<grid, kThreads, 0, st>>>(mp);
    if (rc_status s = check_launch("rc_match_blocks_layer_mean(tiles)")) return s;
    const dim3 sgrid((unsigned)((Q + 63) / 64), (unsigned)nchunks);
    tile_sums_select_kernel<<<sgrid, 256, 0, st>>>(dpart, ls.groups, (int)P, (int)Q, (int)npt, (int)nqt, sel_rows, scale, 0,
                                                    pool_live, part);
    if (rc_status s = check_launch("rc_match_blocks_layer_mean(select)")) return s;
  }
  layer_mean_finalize_kernel<<<(unsigned)((Q + 63) / 64), 256, 0, st>>>(part, (int)nchunks, (int)Q, threshold, best_idx,
                                                                        best_dist, match_idx, second_dist);
  return check_launch("rc_match_blocks_layer_mean(finalize)");
}
