// Attention kernel for small and medium active sets: the NW (4 or 8) wavefronts of a workgroup split the keys.
// Included by attention.hip (uses its helpers).
//
// Work item = (sequence, kv head, group of NQ query tiles of 16 rows, key slice). The workgroup's key
// tiles (32 keys each) are dealt round-robin to its wavefronts; every wavefront streams its tiles through a
// private LDS region (K and V rows as stored; the V operand of the second product comes out of LDS through
// transposing reads; the next tile's global loads are in flight during the products) and keeps an online softmax for its NQ query tiles. At the end the NW
// (max, sum, unnormalised output) states meet in LDS and are merged there, so with one key slice per item the
// normalised bf16 output is written directly: no partial records in global memory and no merge launch. With
// several key slices the merged state of the workgroup is one partial record (a quarter of what one record
// per wavefront would need) for attn_merge.
//
// FUSE: the cache update of the step (Eq. 4: the rows of M_{t-1} are replaced by the freshly computed ones)
// happens inside this kernel instead of in a launch before it. Every lane holds one active position of the
// sequence (at most 64 rows per sequence); after a tile of cache rows has been staged in LDS, the tile's
// active rows are overwritten there with the new K/V rows, and the workgroups of query group 0 also write
// them to the cache in global memory. Workgroups that read such a row from global memory while it is being
// written replace it in LDS anyway, so no ordering between workgroups is needed.
#pragma once

template <int DH, int NQ, int NW, bool FUSE>
__global__ __launch_bounds__(64 * NW, 8 / NW) void attn_bf16_ksplit(
    const bf16_t *__restrict__ Q, bf16_t *Kc, bf16_t *Vc, const int *__restrict__ row_off,
    bf16_t *__restrict__ out, float *__restrict__ part, int batch, int Hq, int Hkv, int L, int q_groups,
    int splits, int tiles_per_split, int rows_cap, float scale_log2e, const bf16_t *__restrict__ k_new,
    const bf16_t *__restrict__ v_new, const int *__restrict__ active_idx) {
    using SM = AttnSmem<DH>;
    constexpr int REC = DH + 4;                       // floats per merged row: m, l, pad, pad, o[DH]
    static_assert(NQ * 16 * REC * 4 <= SM::WAVE_BYTES, "merge records fit the wavefront's LDS region");
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    unsigned char *ksm = smem_raw + wave * SM::WAVE_BYTES;
    unsigned char *vsm = ksm + SM::K_BYTES;

    const int G = Hq / Hkv;
    int pair, within;
    if (!attn_item(blockIdx.x, batch * Hkv, q_groups * splits, pair, within)) return;
    const int split = within % splits, qg = within / splits;
    const int kvh = pair % Hkv, b = pair / Hkv;

    const int qi = lane & 15, g = lane >> 4;
    bf16_t *Kb = Kc + ((size_t)b * Hkv + kvh) * (size_t)L * DH;
    bf16_t *Vb = Vc + ((size_t)b * Hkv + kvh) * (size_t)L * DH;
    const int n_tiles = (L + KT - 1) / KT;
    const int t_begin = split * tiles_per_split, t_end = min(n_tiles, t_begin + tiles_per_split);

    constexpr int KCH = KT * DH / 8 / 64;             // 16-byte chunks of K (and of V) per lane
    uint4 kreg[KCH], vreg[KCH];
    // chunk i of a lane: key lane / (DH/8) + i * 64 / (DH/8) of the tile, dims [8 (lane % (DH/8)), +8)
    constexpr int ROWS_PER_I = 64 / (DH / 8);
    const int lane_off = (lane / (DH / 8)) * DH + (lane % (DH / 8)) * 8;
    // One query group per (sequence, kv head): nobody else reads these K/V rows in this launch, so they are
    // fetched with the non-temporal hint; with several query groups the rows are meant to be found in L2 again.
    const bool read_once = q_groups == 1;
    auto load_tile = [&](int t) {
        const size_t base = (size_t)t * KT * DH;               // wave-uniform
        const bf16_t *kt = Kb + base + lane_off, *vt = Vb + base + lane_off;
        if ((t + 1) * KT <= L && read_once) {
#pragma unroll
            for (int i = 0; i < KCH; ++i) {
                kreg[i] = load16_nt(kt + i * ROWS_PER_I * DH);
                vreg[i] = load16_nt(vt + i * ROWS_PER_I * DH);
            }
        } else if ((t + 1) * KT <= L) {
#pragma unroll
            for (int i = 0; i < KCH; ++i) {
                kreg[i] = *reinterpret_cast<const uint4 *>(kt + i * ROWS_PER_I * DH);
                vreg[i] = *reinterpret_cast<const uint4 *>(vt + i * ROWS_PER_I * DH);
            }
        } else {
            const int key = t * KT + lane / (DH / 8);
#pragma unroll
            for (int i = 0; i < KCH; ++i) {
                const bool ok = key + i * ROWS_PER_I < L;
                kreg[i] = ok ? *reinterpret_cast<const uint4 *>(kt + i * ROWS_PER_I * DH) : make_uint4(0, 0, 0, 0);
                vreg[i] = ok ? *reinterpret_cast<const uint4 *>(vt + i * ROWS_PER_I * DH) : make_uint4(0, 0, 0, 0);
            }
        }
    };
    unsigned char *k_dst = ksm + (lane / (DH / 8)) * SM::K_STRIDE + (lane % (DH / 8)) * 16;
    unsigned char *v_dst = vsm + (lane / (DH / 8)) * SM::V_STRIDE + (lane % (DH / 8)) * 16;
    auto store_tile = [&]() {
#pragma unroll
        for (int i = 0; i < KCH; ++i) {
            *reinterpret_cast<uint4 *>(k_dst + i * ROWS_PER_I * SM::K_STRIDE) = kreg[i];
            *reinterpret_cast<uint4 *>(v_dst + i * ROWS_PER_I * SM::V_STRIDE) = vreg[i];
        }
    };
    const unsigned char *vrow0 = vsm + (4 * g + (qi >> 2)) * SM::V_STRIDE + (qi & 3) * 8;

    float m_run[NQ];
    f32x4 acc[NQ][DH / 16], l_acc[NQ];
    const bf16x8 ones = row_sum_operand(lane);
#pragma unroll
    for (int j = 0; j < NQ; ++j) {
        m_run[j] = -INFINITY;
        l_acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int i = 0; i < DH / 16; ++i) acc[j][i] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    // this wavefront's tiles: t_begin + wave, + NW, + 2 NW, ...
    // The first tile's loads are issued before the row offsets and the query rows are fetched: the K/V addresses do
    // not depend on them, so the memory latencies overlap instead of adding up (the kernel is latency-bound at small
    // active sets). A workgroup that turns out to have no query rows has fetched a tile for nothing.
    int t = t_begin + wave;
    if (t < t_end) load_tile(t);

    const int r0 = row_off[b], nrows = row_off[b + 1] - r0;
    const int nq = nrows * G;                    // query rows of this (sequence, kv head)
    const int m0 = qg * NQ * 16;
    if (m0 >= nq) return;                        // uniform for the workgroup: no barrier is skipped by part of it
    int my_pos = -1;                             // FUSE: active position number `lane` of this sequence
    if (FUSE && lane < nrows && r0 + lane < rows_cap) my_pos = active_idx[r0 + lane];
    bf16x8 qf[NQ][DH / 32];
#pragma unroll
    for (int j = 0; j < NQ; ++j) {
        const int mq = m0 + 16 * j + qi;
        // rows beyond the host's bound have no slot in the output or partial buffers
        const bool ok = mq < nq && r0 + mq / G < rows_cap;
        const bf16_t *qp = Q + ((size_t)(ok ? r0 + mq / G : 0) * Hq + kvh * G + (ok ? mq % G : 0)) * DH + 8 * g;
#pragma unroll
        for (int ks = 0; ks < DH / 32; ++ks) {
            uint4 v = ok ? *reinterpret_cast<const uint4 *>(qp + 32 * ks) : make_uint4(0, 0, 0, 0);
            qf[j][ks] = *reinterpret_cast<bf16x8 *>(&v);
        }
    }

    for (; t < t_end; t += NW) {
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        store_tile();
        if (FUSE) {
            unsigned long long hit = __ballot(my_pos >= t * KT && my_pos < (t + 1) * KT);
            while (hit) {                                    // wave-uniform: rows of this tile that are replaced
                const int src = __ffsll(hit) - 1;
                hit &= hit - 1;
                const int p = __shfl(my_pos, src, 64);
                if (lane < 2 * (DH / 8)) {                   // 16-byte chunks: first the K row, then the V row
                    const bool is_v = lane >= DH / 8;
                    const int ch = lane % (DH / 8);
                    const size_t row = ((size_t)(r0 + src) * Hkv + kvh) * DH + ch * 8;
                    const uint4 v = *reinterpret_cast<const uint4 *>((is_v ? v_new : k_new) + row);
                    *reinterpret_cast<uint4 *>((is_v ? vsm + (p - t * KT) * SM::V_STRIDE
                                                     : ksm + (p - t * KT) * SM::K_STRIDE) + ch * 16) = v;
                    if (qg == 0) *reinterpret_cast<uint4 *>((is_v ? Vb : Kb) + (size_t)p * DH + ch * 8) = v;
                }
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        if (t + NW < t_end) load_tile(t + NW);

        f32x4 st[NQ][2];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const unsigned char *krow = ksm + (16 * h + qi) * SM::K_STRIDE + g * 16;
#pragma unroll
            for (int j = 0; j < NQ; ++j) st[j][h] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < DH / 32; ++ks) {
                const bf16x8 kf = *reinterpret_cast<const bf16x8 *>(krow + ks * 64);
#pragma unroll
                for (int j = 0; j < NQ; ++j)
                    st[j][h] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf, qf[j][ks], st[j][h], 0, 0, 0);
            }
        }
        // st[j][h][i] is the score of key 16h + 4g + i of this tile against query qi of tile j
        bf16x8 pb[NQ][1];
#pragma unroll
        for (int j = 0; j < NQ; ++j)
            softmax_step<2, DH / 16>(st[j], m_run[j], l_acc[j], acc[j], pb[j], t * KT + 4 * g, L, (t + 1) * KT > L,
                                     scale_log2e);
#pragma unroll
        for (int j = 0; j < NQ; ++j)
            l_acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, pb[j][0], l_acc[j], 0, 0, 0);
#pragma unroll
        for (int mt = 0; mt < DH / 16; ++mt) {
            const bf16x8 av = vt_operand(vrow0, mt, SM::V_STRIDE, 0);
#pragma unroll
            for (int j = 0; j < NQ; ++j)
                acc[j][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, pb[j][0], acc[j][mt], 0, 0, 0);
        }
    }

    // Each wavefront leaves its state in its own LDS region: record (tile j, query qi) = m, l, -, -, o[DH].
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    float *my_rec = reinterpret_cast<float *>(ksm);
#pragma unroll
    for (int j = 0; j < NQ; ++j) {
        const float l = query_lanes_sum(l_acc[j][0]);
        float *rec = my_rec + (j * 16 + qi) * REC;
        if (g == 0) {
            rec[0] = m_run[j];
            rec[1] = l;
        }
#pragma unroll
        for (int mt = 0; mt < DH / 16; ++mt) *reinterpret_cast<f32x4 *>(rec + 4 + 16 * mt + 4 * g) = acc[j][mt];
    }
    __syncthreads();

    // Merge: thread handles (query row, 4 consecutive output dims) pairs.
    constexpr int CHUNKS = DH / 4;
    for (int idx = tid; idx < NQ * 16 * CHUNKS; idx += 64 * NW) {
        const int qr = idx / CHUNKS, ch = idx % CHUNKS;     // qr = 16 j + qi
        const int mq = m0 + qr;
        if (mq >= nq || r0 + mq / G >= rows_cap) continue;
        float mw[NW], M = -INFINITY;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            mw[w] = reinterpret_cast<const float *>(smem_raw + w * SM::WAVE_BYTES)[qr * REC];
            M = fmaxf(M, mw[w]);
        }
        float lsum = 0.f;
        f32x4 o = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            const float *rec = reinterpret_cast<const float *>(smem_raw + w * SM::WAVE_BYTES) + qr * REC;
            const float wgt = mw[w] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(mw[w] - M);
            lsum += wgt * rec[1];
            o += wgt * *reinterpret_cast<const f32x4 *>(rec + 4 + 4 * ch);
        }
        const size_t pair = (size_t)(r0 + mq / G) * Hq + kvh * G + mq % G;
        if (splits == 1) {
            const float inv = 1.f / lsum;
            uint2 wv;
            wv.x = (uint32_t)f2bf(o[0] * inv) | ((uint32_t)f2bf(o[1] * inv) << 16);
            wv.y = (uint32_t)f2bf(o[2] * inv) | ((uint32_t)f2bf(o[3] * inv) << 16);
            *reinterpret_cast<uint2 *>(out + pair * DH + 4 * ch) = wv;
        } else {
            float *rec = part + (pair * splits + split) * REC;
            if (ch == 0) {
                rec[0] = M;
                rec[1] = lsum;
            }
            *reinterpret_cast<f32x4 *>(rec + 4 + 4 * ch) = o;
        }
    }
}
