// S3 + S4 fused: radial weights are produced on the matrix cores and consumed by the tensor-product messages
// without ever being written to HBM.
//
//   a[j] = nbar^-1/2 sum_{k: dst(k)=j} sum_p w_k[p][c] (C_p . h_src(k) . Yhat(rhat_k)),
//   w_k[p][c] = fc(d_k) alpha_p (W_r2 SiLU(W_r1 B(d_k)))[p*E + c]
// (Sec. 3 "Message passing"; coupling of Sec. 2.2 / Eq. 1 in the bond frame of Sec. 2.1 / Fig. 2(d)).
//
// Three kernels.  (1) The hidden activations of every edge (times the cutoff envelope) are computed once, cut into
// bf16 pieces and stored in the register layout of the MFMA A operand, one 12 KB record per 32 consecutive edges.
// (2) The rows of the pre-split W_r2 are re-ordered into the layout of the B operand, per group of 8 channels.
// (3) The main kernel: one workgroup per destination node and group of 8 channels, the node's edges in tiles of 128
// (four 32-edge records, aligned to the records of (1)).  The tile is 128 edges x 8 channels rather than 32 x 32
// because every tile streams the whole B operand of its channels through the CU's vector memory path; the narrow
// channel group makes that stream four times shorter per edge-channel.
//
// The eight waves are specialised and run as a two-stage pipeline over the chunks of the product (a chunk = all
// coupling paths with the same input degree l1; it uses a contiguous run of weights and one degree block of the
// source features):
//   producers (waves 0-3): wave (rp, cj) owns the edge records 2 rp, 2 rp + 1 of the tile (A operand in registers for
//     the whole tile) and every second 32-column block of a chunk.  A "slot" is one column block against both
//     records: 48 split-bf16 MFMAs (six products per fp32 product).  Operand registers are refilled in place: as
//     soon as the MFMAs of one k-step have been issued, the loads that bring the same k-step of the next slot
//     (for the A operand: of the next tile) are issued, so nothing is double-buffered and every load has three
//     quarters of a slot to arrive.  The 128 x (paths of the chunk) x 8 weights go to one of two LDS buffers;
//   consumers (waves 4-7): lane = (edge slot, channel), four edges of the tile per lane.  While the producers
//     fill one buffer they read the other: rotate the degree-l1 block of the source row (prefetched during the
//     previous step) into the bond frame, run the chunk of the product, keep the bond-frame result of each edge
//     in registers; after the last chunk the result is rotated back and added to the lane's partial node sum.
// One workgroup barrier per chunk; the fences around it cover LDS only, so loads that prefetch operands for
// later steps stay in flight across it.  Slots are added in fixed order through LDS at the end:
// deterministic, no atomics.
//
// Status: correct (parity-tested at every supported shape, full sizes included) but opt-in (EGNN_OPT_FUSED): at
// 3,000 atoms / 32 channels / l_max 4 it takes 1.5 ms against 0.75 + 0.58 ms for the two-kernel route.  Measured
// with per-barrier timestamps: a producer slot (48 MFMAs) takes 2,200 cycles against 1,536 of pure pipe time; a
// consumer step carries about 3,000 cycles of exposed latency on top of its ALU work, because a single consumer wave
// per SIMD has nothing to switch to while it waits on LDS; and with one MFMA stream and one ALU stream on a SIMD the
// two overlap only partly (a two-wave test loop reaches 1.4x the serial rate, not 2x).  That puts the floor of this
// design near 0.9 ms; what would get it there: edge data of the next tile loaded a chunk earlier (the last chunk
// of a tile stalls 4,000 cycles on it), LDS operands of the next edge prefetched in the consumer.
#include "egnn_internal.h"
#include "bond_frame.h"
#include "split_bf16.h"

#define FP_TILE 128      // edges per tile: one 32-row MFMA block per producer wave
#define FP_CG 8          // channels per workgroup
#define FP_THREADS 512
#define FP_SLOTS 32      // consumer edge slots: 256 lanes / FP_CG
#define FP_PAIRS 4       // edges of a tile per consumer lane
#define FP_TRIG 20       // floats per edge of staged cos/sin (16 used); 80-byte rows spread over the banks

template <int LMAX>
struct FpCfg {
  using Mid = typename LayerMid<LMAX>::T;
  static constexpr int D = (LMAX + 1) * (LMAX + 1);
  static constexpr int NCHUNK = LMAX + 1;
  // weights of a chunk per (edge, channel): padded to an odd number of float4, which makes both the producers'
  // scalar writes and the consumers' 128-bit reads free of bank conflicts
  static constexpr int WQ = ((Mid::CHUNK_MAX + 3) / 4) | 1;
  static constexpr int WPAD = 4 * WQ;
  static constexpr int SWLD = FP_CG * WPAD;        // floats per edge row
  static constexpr int BUF = FP_TILE * SWLD;       // floats per weight buffer
  static constexpr int RED = FP_SLOTS * D * FP_CG; // floats of the slot reduction
  // 32-column MFMA blocks of chunk l1, and the index of its first block in the packed operand
  static constexpr int blocks_of(int l1) { return (Mid::CHUNK_COUNT[l1] * FP_CG + 31) / 32; }
  static constexpr int first_block(int l1) {
    int s = 0;
    for (int i = 0; i < l1; ++i) s += blocks_of(i);
    return s;
  }
  static constexpr int NBLK = first_block(LMAX + 1);
  // producer slots (one column block per producer parity) of chunk l1, and the index of its first slot in a tile
  static constexpr int slots_of(int l1) { return (blocks_of(l1) + 1) / 2; }
  static constexpr int first_slot(int l1) {
    int s = 0;
    for (int i = 0; i < l1; ++i) s += slots_of(i);
    return s;
  }
  static constexpr int NSLOT = first_slot(LMAX + 1);
};

struct FpArgs {
  const int* row_ptr;
  const int* src;
  const float4* rhat_d;
  const float* h;
  const float* W_r1;
  const uint4* W2f;     // packed B operand, see fp_pack_kernel
  const uint4* Af;      // A operand records, see fp_hidden_kernel
  float* a;
  int n_owned, nodes_per_xcd, n_rbf, log2E, n_cg, n_rec;
  float scale, r_cut;
};

__device__ __forceinline__ void fp_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// ---------------------------------------------------------------------------------------------- producers
// The B operand in the order the producers read it: [channel group][block][i = piece*4 + step][lane] uint4, so that
// each of the 12 loads of a block is one contiguous kilobyte over the wave.  Column cc = NBI*32 + (lane & 31) of chunk
// L1 <-> (path cc / 8 of the chunk, channel cc % 8); columns past the chunk repeat a valid row (never stored).
struct FpPackTab {
  int first_path[16], n_paths[16], nbi[16];   // per block
  int n_blocks;
};

__global__ __launch_bounds__(256) void fp_pack_kernel(const uint4* __restrict__ W2s, uint4* __restrict__ W2f,
                                                      FpPackTab tab, int log2E, int n_cg) {
  const int idx = blockIdx.x * 256 + threadIdx.x;
  const int lane = idx & 63, i = (idx >> 6) % 12, blk = (idx / 768) % tab.n_blocks, cg = idx / (768 * tab.n_blocks);
  if (cg >= n_cg) return;
  const int m = lane & 31, hh = lane >> 5, p = i >> 2, t = i & 3;
  const int cc = tab.nbi[blk] * 32 + m;
  const int pi = cc >> 3, ch = cc & 7;
  const int n = (((pi < tab.n_paths[blk]) ? tab.first_path[blk] + pi : tab.first_path[blk]) << log2E) + cg * FP_CG + ch;
  W2f[idx] = W2s[(size_t)n * 24 + p * 8 + hh * 4 + t];   // a row of the split W_r2: [3 pieces][64 units] bf16 = 24 uint4
}

// Chunk and position inside it of producer slot S of a tile.
template <int LMAX, int S>
struct FpSlot {
  using Cfg = FpCfg<LMAX>;
  static constexpr int chunk() {
    int l1 = 0;
    while (Cfg::first_slot(l1 + 1) <= S) ++l1;
    return l1;
  }
  static constexpr int L1 = chunk();
  static constexpr int I = S - Cfg::first_slot(L1);
  static constexpr int NB = Cfg::blocks_of(L1);
  static constexpr bool LAST_OF_CHUNK = I + 1 == Cfg::slots_of(L1);
};

// hidden activations (times the cutoff envelope) of an edge of length d, units hh*32 .. hh*32+31, as the A operand
// in pieces: a[piece*4 + t] holds units hh*32 + 8t .. +7
__device__ __forceinline__ void fp_hidden(const float* sW1, int n_rbf, float r_cut, float d, int hh, uint4 (&a)[12]) {
  const float step = r_cut / (float)(n_rbf - 1);
  const float inv2s2 = 0.5f / (step * step);
  float pre[32];
#pragma unroll
  for (int s = 0; s < 32; ++s) pre[s] = 0.0f;
  for (int b = 0; b < n_rbf; ++b) {
    const float u = d - (float)b * step;
    const float B = __expf(-u * u * inv2s2);
    const float* wrow = sW1 + b * EGNN_HIDDEN + hh * 32;
#pragma unroll
    for (int s = 0; s < 32; ++s) pre[s] += wrow[s] * B;
  }
  const float fc = egnn_envelope(d, r_cut);
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    uint32_t ph[4], pm[4], pl[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const float x0 = pre[8 * t + 2 * q], x1 = pre[8 * t + 2 * q + 1];
      const Split3 s0 = split3(fc * x0 / (1.0f + __expf(-x0)));
      const Split3 s1 = split3(fc * x1 / (1.0f + __expf(-x1)));
      ph[q] = pack2(s0.hi, s1.hi);
      pm[q] = pack2(s0.mid, s1.mid);
      pl[q] = pack2(s0.lo, s1.lo);
    }
    a[0 * 4 + t] = make_uint4(ph[0], ph[1], ph[2], ph[3]);
    a[1 * 4 + t] = make_uint4(pm[0], pm[1], pm[2], pm[3]);
    a[2 * 4 + t] = make_uint4(pl[0], pl[1], pl[2], pl[3]);
  }
}

// A operand records: Af[record][i = piece*4 + step][lane] uint4, record q = edges 32 q .. 32 q + 31 (the last one
// repeats the last edge), lane = (edge & 31) + 32 * half of the hidden units.  One wave per record.
__global__ __launch_bounds__(256) void fp_hidden_kernel(const float4* __restrict__ rhat_d, long n_edges,
                                                        const float* __restrict__ W_r1, uint4* __restrict__ Af,
                                                        int n_rec, int n_rbf, float r_cut) {
  __shared__ float sW1[32 * EGNN_HIDDEN];
  for (int i = threadIdx.x; i < n_rbf * EGNN_HIDDEN; i += 256) sW1[i] = W_r1[(i & 63) * n_rbf + (i >> 6)];
  __syncthreads();
  const int lane = threadIdx.x & 63;
  const int q = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (q >= n_rec) return;
  long e = (long)q * 32 + (lane & 31);
  if (e >= n_edges) e = n_edges - 1;
  uint4 a[12];
  fp_hidden(sW1, n_rbf, r_cut, rhat_d[e].w, lane >> 5, a);
  uint4* out = Af + (size_t)q * 768 + lane;
#pragma unroll
  for (int i = 0; i < 12; ++i) out[i * 64] = a[i];
}

// source index and cos/sin(m phi), cos/sin(m theta), m = 1..4, of edge r of a tile -> LDS (threads 0..127)
__device__ __forceinline__ void fp_stage_meta(const float4 rd, int sidx, int r, int* ssrc, float* strig) {
  ssrc[r] = sidx;
  BondTrig t;
  egnn_bond_trig<4>(rd.x, rd.y, rd.z, t);
  float4* row = reinterpret_cast<float4*>(strig + r * FP_TRIG);
  row[0] = make_float4(t.cp[1], t.cp[2], t.cp[3], t.cp[4]);
  row[1] = make_float4(t.sp[1], t.sp[2], t.sp[3], t.sp[4]);
  row[2] = make_float4(t.ct[1], t.ct[2], t.ct[3], t.ct[4]);
  row[3] = make_float4(t.st[1], t.st[2], t.st[3], t.st[4]);
}

// What a producer wave needs for one tile.
template <int LMAX>
struct FpProd {
  const FpArgs& g;
  const uint4* w2f_lane;   // packed B operand of this channel group + lane
  const uint4* w2f_next;   // the same for the channel group of the next tile
  const uint4* af_next0;   // A records of this wave in the next tile + lane (valid if has_next)
  const uint4* af_next1;
  float* swrows;           // this wave's first row (record 2 rp) in weight buffer 0
  int* ssrc;
  float* strig;
  int k0, k1, base_next;   // node's edge range; first edge index of the next tile
  int t, tid, lane, cj;    // t: running tile index over (channel group, tile of the node)
  bool has_next;
};

// One slot: column block min(2 I + cj, NB - 1) of chunk L1 against both records of the wave (a wave without a block of
// its own in the last slot of an odd chunk repeats the last block and stores nothing: the step is as long anyway).
template <int LMAX, int S>
__device__ __forceinline__ void fp_slot(const FpProd<LMAX>& cx, uint4 (&a0)[12], uint4 (&a1)[12], uint4 (&b)[12]) {
  using Cfg = FpCfg<LMAX>;
  using Sl = FpSlot<LMAX, S>;
  using Nx = FpSlot<LMAX, (S + 1) % Cfg::NSLOT>;
  constexpr bool LAST = S + 1 == Cfg::NSLOT;
  constexpr int NCH = Cfg::Mid::CHUNK_COUNT[Sl::L1];
  const int m = cx.lane & 31, hh = cx.lane >> 5;
  const int want = 2 * Sl::I + cx.cj;
  const int nbi = want < Sl::NB ? want : Sl::NB - 1;
  const int want_n = 2 * Nx::I + cx.cj;
  const uint4* bnext = (LAST ? cx.w2f_next : cx.w2f_lane) + (Cfg::first_block(Nx::L1) + (want_n < Nx::NB ? want_n : Nx::NB - 1)) * 768;

  // edge data of the next tile for the consumers: loads issued before the last chunk's matrix work, used after it
  constexpr bool STAGE = Sl::L1 == LMAX && Sl::I == 0;
  float4 rd = make_float4(0.f, 0.f, 1.f, 0.f);
  int sidx = 0;
  const bool stage = STAGE && cx.has_next && cx.tid < FP_TILE;
  if (STAGE && stage) {
    int k = cx.base_next + cx.tid;
    k = k < cx.k0 ? cx.k0 : (k < cx.k1 ? k : cx.k1 - 1);
    rd = cx.g.rhat_d[k];
    sidx = cx.g.src[k];
  }

  float16v acc0, acc1;
#pragma unroll
  for (int i = 0; i < 16; ++i) acc0[i] = acc1[i] = 0.0f;
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    // smallest terms first: (lo,hi) (hi,lo) (mid,mid) (mid,hi) (hi,mid) (hi,hi); the two records alternate
    constexpr int pa[6] = {2, 0, 1, 1, 0, 0};
    constexpr int pb[6] = {0, 2, 1, 0, 1, 0};
#pragma unroll
    for (int q = 0; q < 6; ++q) {
      acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(a0[pa[q] * 4 + t]), as_bf16x8(b[pb[q] * 4 + t]), acc0, 0, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(a1[pa[q] * 4 + t]), as_bf16x8(b[pb[q] * 4 + t]), acc1, 0, 0, 0);
    }
    __builtin_amdgcn_sched_barrier(0);   // the refills below stay behind the MFMAs that read the registers ...
#pragma unroll
    for (int p = 0; p < 3; ++p) b[p * 4 + t] = bnext[(p * 4 + t) * 64];
    if (LAST && cx.has_next) {
#pragma unroll
      for (int p = 0; p < 3; ++p) {
        a0[p * 4 + t] = cx.af_next0[(p * 4 + t) * 64];
        a1[p * 4 + t] = cx.af_next1[(p * 4 + t) * 64];
      }
    }
    __builtin_amdgcn_sched_barrier(0);   // ... and ahead of the next k-step
  }
  const int cc = nbi * 32 + m;
  const int pi = cc >> 3, ch = cc & 7;
  if (want < Sl::NB && pi < NCH) {
    const int step = cx.t * Cfg::NCHUNK + Sl::L1;
    float* col = cx.swrows + (step & 1) * Cfg::BUF + ch * Cfg::WPAD + pi;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int row = 8 * (i >> 2) + 4 * hh + (i & 3);
      col[row * Cfg::SWLD] = acc0[i];
      col[(32 + row) * Cfg::SWLD] = acc1[i];
    }
  }
  if (STAGE && stage)
    fp_stage_meta(rd, sidx, cx.tid, cx.ssrc + ((cx.t + 1) & 1) * FP_TILE, cx.strig + ((cx.t + 1) & 1) * FP_TILE * FP_TRIG);
  if constexpr (Sl::LAST_OF_CHUNK) fp_barrier();
  __builtin_amdgcn_sched_barrier(0);
  if constexpr (!LAST) fp_slot<LMAX, S + 1>(cx, a0, a1, b);
}

// ---------------------------------------------------------------------------------------------- consumers
__device__ __forceinline__ void fp_read_trig(const float* strig, int r, BondTrig& t) {
  const float4* row = reinterpret_cast<const float4*>(strig + r * FP_TRIG);
  const float4 a = row[0], b = row[1], c = row[2], d = row[3];
  t.cp[0] = 1.0f; t.sp[0] = 0.0f; t.ct[0] = 1.0f; t.st[0] = 0.0f;
  t.cp[1] = a.x; t.cp[2] = a.y; t.cp[3] = a.z; t.cp[4] = a.w;
  t.sp[1] = b.x; t.sp[2] = b.y; t.sp[3] = b.z; t.sp[4] = b.w;
  t.ct[1] = c.x; t.ct[2] = c.y; t.ct[3] = c.z; t.ct[4] = c.w;
  t.st[1] = d.x; t.st[2] = d.y; t.st[3] = d.z; t.st[4] = d.w;
}

// degree-L1 block of the source rows of this lane's edges (every staged row holds a valid source index)
template <int LMAX, int L1>
__device__ __forceinline__ void fp_gather(const FpArgs& g, const int* ssrc, int slot, int chan,
                                          float (&v)[FP_PAIRS][2 * L1 + 1]) {
  constexpr int D = FpCfg<LMAX>::D;
#pragma unroll
  for (int q = 0; q < FP_PAIRS; ++q) {
    const float* hp = g.h + (((size_t)ssrc[slot + FP_SLOTS * q] * D + L1 * L1) << g.log2E) + chan;
#pragma unroll
    for (int i = 0; i < 2 * L1 + 1; ++i) v[q][i] = hp[(size_t)i << g.log2E];
  }
}

// rows r of the tile with lo <= r < hi are edges of the node
template <int LMAX, int L1>
__device__ __forceinline__ void fp_consume(const float* swbuf, const float* strig, int lo, int hi, int slot, int c,
                                           const float (&v)[FP_PAIRS][2 * L1 + 1],
                                           float (&o)[FP_PAIRS][FpCfg<LMAX>::D]) {
  using Cfg = FpCfg<LMAX>;
  constexpr int NCH = Cfg::Mid::CHUNK_COUNT[L1];
  constexpr int NQ = (NCH + 3) / 4;
#pragma unroll
  for (int q = 0; q < FP_PAIRS; ++q) {
    const int r = slot + FP_SLOTS * q;
    if (r >= lo && r < hi) {
      float wl[4 * NQ], vv[2 * L1 + 1];
      const float4* wp = reinterpret_cast<const float4*>(swbuf + r * Cfg::SWLD + c * Cfg::WPAD);
#pragma unroll
      for (int i = 0; i < NQ; ++i) {
        const float4 x = wp[i];
        wl[4 * i] = x.x; wl[4 * i + 1] = x.y; wl[4 * i + 2] = x.z; wl[4 * i + 3] = x.w;
      }
#pragma unroll
      for (int i = 0; i < 2 * L1 + 1; ++i) vv[i] = v[q][i];
      if constexpr (L1 > 0) {
        BondTrig t;
        fp_read_trig(strig, r, t);
        egnn_to_bond_frame_l<L1>(vv, t);
      }
      Cfg::Mid::template run_l1<L1>(vv, wl, o[q]);
    }
  }
}

// after the last chunk of a tile: back to the lab frame, into the node's partial sums; o is cleared for the next tile
template <int LMAX>
__device__ __forceinline__ void fp_finish_tile(const float* strig, int lo, int hi, int slot,
                                               float (&o)[FP_PAIRS][FpCfg<LMAX>::D], float (&acc)[FpCfg<LMAX>::D]) {
  constexpr int D = FpCfg<LMAX>::D;
#pragma unroll
  for (int q = 0; q < FP_PAIRS; ++q) {
    const int r = slot + FP_SLOTS * q;
    if (r >= lo && r < hi) {
      BondTrig t;
      fp_read_trig(strig, r, t);
      egnn_from_bond_frame<LMAX>(o[q], t);
#pragma unroll
      for (int i = 0; i < D; ++i) acc[i] += o[q][i];
    }
#pragma unroll
    for (int i = 0; i < D; ++i) o[q][i] = 0.0f;
  }
}

// Slot sums of one channel group (left in `red` by the consumers before the last barrier) -> node row, fixed order.
template <int LMAX>
__device__ __forceinline__ void fp_flush(const FpArgs& g, const float* red, int j, int cg, int ctid) {
  constexpr int D = FpCfg<LMAX>::D;
  if (ctid < D * FP_CG) {
    float sum = 0.0f;
#pragma unroll 8
    for (int s = 0; s < FP_SLOTS; ++s) sum += red[s * D * FP_CG + ctid];
    g.a[(((size_t)j * D + (ctid >> 3)) << g.log2E) + cg * FP_CG + (ctid & 7)] = sum * g.scale;
  }
}

// One pipeline step of the consumers on chunk L1 of running tile `run`: prefetch the source block of the next chunk
// (of the next tile, possibly of the next channel group, after the last chunk), run this chunk, barrier.
template <int LMAX, int L1, class VCur, class VNext>
__device__ __forceinline__ void fp_consumer_step(const FpArgs& g, const float* sw, const int* ssrc, const float* strig,
                                                 float* red, int run, int lo, int hi, bool has_next, bool last_of_cg,
                                                 int slot, int c, int chan, int chan_next,
                                                 const VCur& vcur, VNext& vnext, float (&o)[FP_PAIRS][FpCfg<LMAX>::D],
                                                 float (&acc)[FpCfg<LMAX>::D]) {
  using Cfg = FpCfg<LMAX>;
  constexpr int D = Cfg::D;
  const int par = run & 1;
  if constexpr (L1 < LMAX) {
    fp_gather<LMAX, L1 + 1>(g, ssrc + par * FP_TILE, slot, chan, vnext);
  } else {
    if (has_next) fp_gather<LMAX, 0>(g, ssrc + (par ^ 1) * FP_TILE, slot, chan_next, vnext);
  }
  const int step = run * Cfg::NCHUNK + L1;
  fp_consume<LMAX, L1>(sw + (step & 1) * Cfg::BUF, strig + par * FP_TILE * FP_TRIG, lo, hi, slot, c, vcur, o);
  if constexpr (L1 == LMAX) {
    fp_finish_tile<LMAX>(strig + par * FP_TILE * FP_TRIG, lo, hi, slot, o, acc);
    if (last_of_cg) {   // the node's sums of this channel group: slots are added after the barrier (fp_flush)
#pragma unroll
      for (int i = 0; i < D; ++i) {
        red[(slot * D + i) * FP_CG + c] = acc[i];
        acc[i] = 0.0f;
      }
    }
  }
  fp_barrier();
}

template <int LMAX>
__global__ __launch_bounds__(FP_THREADS) void layer_fused_kernel(FpArgs g) {
  using Cfg = FpCfg<LMAX>;
  constexpr int D = Cfg::D;
  extern __shared__ float4 smem4[];
  float* sw = reinterpret_cast<float*>(smem4);                 // [2][FP_TILE][SWLD]
  float* strig = sw + 2 * Cfg::BUF;                            // [2][FP_TILE][FP_TRIG]
  float* red = strig + 2 * FP_TILE * FP_TRIG;                  // [FP_SLOTS][D][FP_CG]
  int* ssrc = reinterpret_cast<int*>(red + Cfg::RED);          // [2][FP_TILE]

  // consecutive nodes go to the same XCD, i.e. share an L2
  const int j = (blockIdx.x & 7) * g.nodes_per_xcd + (blockIdx.x >> 3);
  if (j >= g.n_owned) return;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int k0 = g.row_ptr[j], k1 = g.row_ptr[j + 1];
  // tiles are aligned to the 32-edge records of the A operand: tile t = records rec0 + 4 t .. + 3
  const int rec0 = k0 >> 5;
  const int n_tiles = k1 > k0 ? (((k1 + 31) >> 5) - rec0 + 3) >> 2 : 0;
  const int base0 = rec0 << 5;   // edge index of row 0 of tile 0
  if (n_tiles == 0) {            // no incoming edge: the sum is empty
    float* out = g.a + (((size_t)j * D) << g.log2E);
    for (int i = tid; i < (D << g.log2E); i += FP_THREADS) out[i] = 0.0f;
    return;
  }
  // The workgroup walks the channel groups one after the other; (channel group, tile) pairs form one running
  // sequence of tiles, so the pipeline never drains between channel groups.
  const int n_run = g.n_cg * n_tiles;

  if (tid < FP_TILE) {
    int k = base0 + tid;
    k = k < k0 ? k0 : (k < k1 ? k : k1 - 1);
    fp_stage_meta(g.rhat_d[k], g.src[k], tid, ssrc, strig);
  }
  fp_barrier();

  if (wave < 4) {
    // ------------------------------------------------------------------------------------------ producer
    const int rp = wave >> 1, cj = wave & 1;
    uint4 a0[12], a1[12], b[12];
    // an offset the compiler cannot see through: the operands repeat from tile to tile, and without this
    // their loads are hoisted out of the tile loop (they would not fit the register file)
    int zero = 0;
    asm volatile("" : "+s"(zero));
    const int last_rec = g.n_rec - 1;
    {
      const int q0 = rec0 + 2 * rp, q1 = q0 + 1;
      const uint4* p0 = g.Af + (size_t)(q0 < last_rec ? q0 : last_rec) * 768 + lane + zero;
      const uint4* p1 = g.Af + (size_t)(q1 < last_rec ? q1 : last_rec) * 768 + lane + zero;
      const uint4* pb = g.W2f + lane + zero + (Cfg::first_block(0) + (cj < Cfg::blocks_of(0) ? cj : Cfg::blocks_of(0) - 1)) * 768;
#pragma unroll
      for (int i = 0; i < 12; ++i) {
        a0[i] = p0[i * 64];
        a1[i] = p1[i * 64];
        b[i] = pb[i * 64];
      }
    }
    int cg = 0, t = 0;
    for (int run = 0; run < n_run; ++run) {
      asm volatile("" : "+s"(zero));
      int cg_n = cg, t_n = t + 1;
      if (t_n == n_tiles) { t_n = 0; ++cg_n; }
      const int q0 = rec0 + 4 * t_n + 2 * rp, q1 = q0 + 1;
      FpProd<LMAX> cx{g,
                      g.W2f + (size_t)cg * Cfg::NBLK * 768 + lane + zero,
                      g.W2f + (size_t)(cg_n < g.n_cg ? cg_n : cg) * Cfg::NBLK * 768 + lane + zero,   // (refilled even after the last tile)
                      g.Af + (size_t)(q0 < last_rec ? q0 : last_rec) * 768 + lane + zero,
                      g.Af + (size_t)(q1 < last_rec ? q1 : last_rec) * 768 + lane + zero,
                      sw + (size_t)(rp * 64) * Cfg::SWLD,
                      ssrc, strig, k0, k1, base0 + t_n * FP_TILE, run, tid, lane, cj, run + 1 < n_run};
      fp_slot<LMAX, 0>(cx, a0, a1, b);
      cg = cg_n;
      t = t_n;
    }
    fp_barrier();   // the consumers' last step
  } else {
    // ------------------------------------------------------------------------------------------ consumer
    const int ctid = tid - 256;
    const int c = ctid & (FP_CG - 1), slot = ctid >> 3;
    float acc[D], o[FP_PAIRS][D];
#pragma unroll
    for (int i = 0; i < D; ++i) acc[i] = 0.0f;
#pragma unroll
    for (int q = 0; q < FP_PAIRS; ++q)
#pragma unroll
      for (int i = 0; i < D; ++i) o[q][i] = 0.0f;
    float v0[FP_PAIRS][1], v1[FP_PAIRS][3], v2[FP_PAIRS][5], v3[FP_PAIRS][7], v4[FP_PAIRS][9];
    fp_gather<LMAX, 0>(g, ssrc, slot, c, v0);
    fp_barrier();   // the producers' first step
    int cg = 0, t = 0;
    int flush_cg = -1;   // channel group whose slot sums wait in `red`
    for (int run = 0; run < n_run; ++run) {
      if (flush_cg >= 0) {   // written before the last barrier; nobody writes `red` again before a whole tile has passed
        fp_flush<LMAX>(g, red, j, flush_cg, ctid);
        flush_cg = -1;
      }
      const int base = base0 + t * FP_TILE;
      const int lo = k0 - base, hi = k1 - base;   // rows lo <= r < hi of the tile belong to the node
      const bool has_next = run + 1 < n_run;
      int cg_n = cg, t_n = t + 1;
      if (t_n == n_tiles) { t_n = 0; ++cg_n; }
      const int chan = cg * FP_CG + c, chan_n = cg_n * FP_CG + c;
#define FP_STEP(L1, VC, VN) \
  fp_consumer_step<LMAX, L1>(g, sw, ssrc, strig, red, run, lo, hi, has_next, t_n == 0, slot, c, chan, chan_n, VC, VN, o, acc);
      if constexpr (LMAX == 1) { FP_STEP(0, v0, v1) FP_STEP(1, v1, v0) }
      if constexpr (LMAX == 2) { FP_STEP(0, v0, v1) FP_STEP(1, v1, v2) FP_STEP(2, v2, v0) }
      if constexpr (LMAX == 3) { FP_STEP(0, v0, v1) FP_STEP(1, v1, v2) FP_STEP(2, v2, v3) FP_STEP(3, v3, v0) }
      if constexpr (LMAX == 4) { FP_STEP(0, v0, v1) FP_STEP(1, v1, v2) FP_STEP(2, v2, v3) FP_STEP(3, v3, v4) FP_STEP(4, v4, v0) }
#undef FP_STEP
      if (t_n == 0) flush_cg = cg;
      cg = cg_n;
      t = t_n;
    }
    fp_flush<LMAX>(g, red, j, flush_cg, ctid);
  }
}

template <int LMAX>
static int launch_fused(egnn_ctx* ctx, FpArgs& args, const void* W2s, int grid, hipStream_t stream) {
  using Cfg = FpCfg<LMAX>;
  using Mid = typename Cfg::Mid;
  static_assert(Cfg::NBLK <= 16, "block table too small");
  FpPackTab tab;
  tab.n_blocks = Cfg::NBLK;
  for (int l1 = 0, blk = 0; l1 <= LMAX; ++l1)
    for (int nbi = 0; nbi < Cfg::blocks_of(l1); ++nbi, ++blk) {
      tab.first_path[blk] = Mid::CHUNK_FIRST[l1];
      tab.n_paths[blk] = Mid::CHUNK_COUNT[l1];
      tab.nbi[blk] = nbi;
    }
  const size_t n_u4 = (size_t)args.n_cg * Cfg::NBLK * 768;
  hipLaunchKernelGGL(fp_pack_kernel, dim3((unsigned)((n_u4 + 255) / 256)), dim3(256), 0, stream,
                     reinterpret_cast<const uint4*>(W2s), const_cast<uint4*>(args.W2f), tab, args.log2E, args.n_cg);
  EGNN_LAUNCH_CHECK(ctx, "fp_pack_kernel");
  const size_t shmem = ((size_t)2 * Cfg::BUF + 2 * FP_TILE * FP_TRIG + Cfg::RED) * sizeof(float) + 2 * FP_TILE * sizeof(int);
  auto kern = layer_fused_kernel<LMAX>;
  if (shmem > 64 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)shmem);
    if (e != hipSuccess) return egnn_check_hip(ctx, e, "hipFuncSetAttribute(layer_fused_kernel)");
  }
  hipLaunchKernelGGL(kern, dim3(grid), dim3(FP_THREADS), shmem, stream, args);
  EGNN_LAUNCH_CHECK(ctx, "layer_fused_kernel");
  return EGNN_OK;
}

bool egnn_fused_supported(const egnn_ctx* ctx) {
  const int E = ctx->desc.channels;
  return ctx->desc.lmax >= 1 && E >= FP_CG && (E & (E - 1)) == 0 && ctx->desc.n_rbf <= 32;
}

// Scratch of the fused route: the packed B operand (upper bound over the supported degrees: 16 blocks of 12 KB per
// channel group), then one 12 KB A record per 32 edges.
static size_t fused_pack_bytes(const egnn_ctx* ctx) { return (size_t)(ctx->desc.channels / FP_CG) * 16 * 768 * sizeof(uint4); }
size_t egnn_fused_scratch_bytes(const egnn_ctx* ctx, int64_t n_edges) {
  return fused_pack_bytes(ctx) + (size_t)((n_edges + 31) / 32) * 768 * sizeof(uint4);
}

// W2s: the pre-split W_r2 (egnn_launch_split_w2); scratch: egnn_fused_scratch_bytes.  a [n_owned][D][E].
int egnn_launch_layer_fused(egnn_ctx* ctx, const egnn_graph* g, const float* rhat_d, const float* h,
                            const float* W_r1, const void* W2s, void* scratch, size_t scratch_bytes, float* a,
                            hipStream_t stream) {
  const int n = g->n_owned;
  if (n == 0) return EGNN_OK;
  if (!egnn_fused_supported(ctx)) return egnn_fail(ctx, EGNN_EINVAL, "layer_fused: unsupported (lmax, channels)");
  if (scratch_bytes < egnn_fused_scratch_bytes(ctx, g->n_edges))
    return egnn_fail(ctx, EGNN_EWS, "layer_fused: scratch too small");
  FpArgs args;
  args.row_ptr = g->row_ptr;
  args.src = g->src;
  args.rhat_d = reinterpret_cast<const float4*>(rhat_d);
  args.h = h;
  args.W_r1 = W_r1;
  args.W2f = reinterpret_cast<const uint4*>(scratch);
  uint4* Af = reinterpret_cast<uint4*>((char*)scratch + fused_pack_bytes(ctx));
  args.Af = Af;
  args.a = a;
  args.n_owned = n;
  args.nodes_per_xcd = (n + 7) / 8;
  args.n_rbf = ctx->desc.n_rbf;
  args.log2E = ctx->log2_channels;
  args.n_cg = ctx->desc.channels / FP_CG;
  args.n_rec = (int)((g->n_edges + 31) / 32);
  args.scale = 1.0f / sqrtf(ctx->desc.agg_norm);
  args.r_cut = ctx->desc.r_cut;
  if (args.n_rec > 0) {
    hipLaunchKernelGGL(fp_hidden_kernel, dim3((args.n_rec + 3) / 4), dim3(256), 0, stream, args.rhat_d, (long)g->n_edges,
                       W_r1, Af, args.n_rec, args.n_rbf, args.r_cut);
    EGNN_LAUNCH_CHECK(ctx, "fp_hidden_kernel");
  }
  const int grid = args.nodes_per_xcd * 8;
  switch (ctx->desc.lmax) {
    case 1: return launch_fused<1>(ctx, args, W2s, grid, stream);
    case 2: return launch_fused<2>(ctx, args, W2s, grid, stream);
    case 3: return launch_fused<3>(ctx, args, W2s, grid, stream);
    case 4: return launch_fused<4>(ctx, args, W2s, grid, stream);
    default: return egnn_fail(ctx, EGNN_EINVAL, "layer_fused: lmax out of range");
  }
}
