// Workgroup-level negacyclic NTT for gfx950: register windows + LDS exchanges.
//
// A workgroup of T = NB / E threads transforms a block of NB = 2^LOGB coefficients that
// is part of a length-2^LOGN transform (LOGB == LOGN: the whole polynomial).  Every thread
// keeps E = 2^ELOG coefficients in registers.  The LOGB butterfly stages are grouped into
// passes of (up to) ELOG stages; during a pass a thread owns the E coefficients whose
// index differs only in the ELOG-bit "window" of that pass, so all butterflies of the
// pass are register-to-register.  Between passes the coefficients change owner through
// LDS (write at the old owner, barrier, read at the new owner); once the window base is 6 or less
// both owners sit in the same wavefront and the barrier is dropped.
//
// Forward transform: merged Cooley-Tukey stages (the psi twist is folded into the
// twiddles), natural-order input, stage s pairs indices that differ in bit LOGN-1-s and
// uses twiddle table entry 2^s + (index >> (LOGN-s)); entry k of the forward table holds
// psi^bitrev(k).  The inverse transform runs Gentleman-Sande stages in the opposite
// order with the inverse table (entry k holds psi^-bitrev(k)) and folds N^-1 into its
// last stage.
//
// Index of a coefficient inside the block during pass p with window base wb:
//     idx = (tid >> wb) << (wb + ELOG) | k << wb | (tid & (2^wb - 1)),   k = register slot.
// Pass 0 has wb = LOGB - ELOG (idx = k * T + tid: coalesced natural order); the last pass
// has wb = 0 (idx = tid * E + k), and evaluation-form data is stored at position
// k * T + tid, so global accesses are coalesced on both sides.
//
// The arithmetic (element type, butterflies, lazy ranges) comes from a policy A (arith.hpp).
#pragma once
#include "arith.hpp"

#ifndef D2_HOST_WAVE_SYNC        // a host build that runs the kernels supplies its own
#define D2_HOST_WAVE_SYNC() __syncthreads()
#endif

namespace d2 {

// Order the LDS accesses of one wavefront: no instruction, only a point the compiler moves no
// memory access across.
D2_DEV void wave_sync()
{
#if D2_GCN_ASM
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#else
    D2_HOST_WAVE_SYNC();
#endif
}

// A line the instruction scheduler moves nothing across (no instruction of its own).
D2_DEV void sched_fence()
{
#if D2_GCN_ASM
    __builtin_amdgcn_sched_barrier(0);
#endif
}

// table entry with an index that is uniform over the workgroup
template <class A>
D2_DEV typename A::Twid load_tw_uniform(const Tw *tw, uint32_t i)
{
    if constexpr (A::SCALAR_TW) return A::load_u(tw, i);
    else return A::load_v(tw, i);
}

template <class A_, int LOGN_, int ELOG_, int LOGB_ = LOGN_>
struct Engine {
    typedef A_ A;
    typedef typename A::elem elem;
    typedef typename A::Mod Mod;
    typedef typename A::Twid Twid;
    static constexpr int LOGN = LOGN_, ELOG = ELOG_, LOGB = LOGB_;
    static constexpr int NB = 1 << LOGB;
    static constexpr int E = 1 << ELOG;
    static constexpr int T = NB / E;
    static constexpr int NPASS = (LOGB + ELOG - 1) / ELOG;
    static constexpr int LDS_WORDS = NB + (NB >> ELOG);   // one pad word per E coefficients
    static constexpr int WAVES = 4;   // waves per SIMD the kernels are compiled for (<= 128 VGPRs)
    // Kernels that run several forward transforms in a row give them two LDS buffers in turn where
    // two fit next to the expected number of resident workgroups (160 KB per CU): the writer of an
    // exchange then never meets a reader of the previous transform, which still works in the other
    // buffer, and the workgroup barrier in front of the write goes away (one barrier per transform
    // instead of two).  Transform n writes buffer n mod 2; its barrier between write and read is
    // reached by every wave only after that wave has finished transform n - 1, hence before any wave
    // starts writing for transform n + 1.
    static constexpr bool PINGPONG = (size_t)LDS_WORDS * 8 * 2 * (T >= 1024 ? 1 : 2) <= 160 * 1024;
    static constexpr int LDS_CHAIN_WORDS = (PINGPONG ? 2 : 1) * LDS_WORDS;
    // the buffer of the next transform of a chain; `turn` starts at 0 when buffer 0 was used last
    D2_DEV static uint64_t *next_buffer(uint64_t *lds, uint32_t &turn)
    {
        if constexpr (PINGPONG) {
            turn ^= 1u;
            return lds + turn * (uint32_t)LDS_WORDS;
        } else {
            return lds;
        }
    }

    static_assert(LOGB >= ELOG && LOGB <= LOGN, "bad engine shape");
    // the same shape (threads, ownership, LDS layout) over another arithmetic: the kernels run their
    // transforms modulo the plaintext modulus with it
    template <class B>
    using Rebind = Engine<B, LOGN_, ELOG_, LOGB_>;

    // number of stages of pass p and the window base
    static constexpr int stages(int p) { return p < NPASS - 1 ? ELOG : LOGB - ELOG * (NPASS - 1); }
    static constexpr int wbase(int p) { return p < NPASS - 1 ? LOGB - ELOG * (p + 1) : 0; }
    // lowest stage bit (position inside the block index) handled by pass p
    static constexpr int sbit(int p) { return p < NPASS - 1 ? wbase(p) : 0; }

    template <int P>
    D2_DEV static int index_of(int k, int tid)
    {
        constexpr int wb = wbase(P);
        return ((tid >> wb) << (wb + ELOG)) | (k << wb) | (tid & ((1 << wb) - 1));
    }

    D2_DEV static int phys(int idx) { return idx + (idx >> ELOG); }

    // position of register slot k of thread tid in evaluation-form storage of the block
    D2_DEV static int eval_pos(int k, int tid) { return k * T + tid; }
    // position in natural (coefficient) order during pass 0
    D2_DEV static int coef_pos(int k, int tid) { return k * T + tid; }

    // Twiddles of a pass: stage bit kb of the window uses E >> (kb + 1) consecutive table entries;
    // they sit in slot (E >> (kb + 1)) - 1 + g of a per-pass array (E - 1 slots for a full window).
    static constexpr int tw_slot(int kb, int g) { return (E >> (kb + 1)) - 1 + g; }
    // With a window base of 6 or more all lanes of a wavefront use the same entries.
    template <int P>
    static constexpr bool uniform_tw() { return A::SCALAR_TW && wbase(P) >= 6; }

    // A pass's twiddles are requested as one set, one pass ahead of their use (the latency then
    // overlaps the butterflies and the exchange in between), if they sit in scalar registers or
    // take at most 32 vector registers; otherwise stage by stage inside the pass.
    template <int P>
    static constexpr bool ahead() { return uniform_tw<P>() || (E - 1) * (int)(sizeof(Twid) / 4) <= 32; }

    // The part of a twiddle index that depends on the thread.
    template <int P>
    D2_DEV static uint32_t tw_hi(int tid)
    {
        constexpr int wb = wbase(P);
        // pass 0: T = 2^wb threads, nothing above the window.  Other uniform passes: taken from
        // the hardware thread id, so that transforms sharing a table also share these loads.
        if constexpr (wb == LOGB - ELOG) return 0;
        else if constexpr (uniform_tw<P>()) return wave_uniform((uint32_t)threadIdx.x >> wb);
        else return (uint32_t)(tid >> wb);
    }

    // Twiddles of the stage with block-index bit B_ of pass P -> DST[OFF_ .. OFF_ + (E >> (kb + 1)));
    // written out where it is used: as a separate function the compiler no longer sees constant
    // array indices and moves the arrays to scratch memory.
#define D2_LOAD_STAGE(DST, OFF_, B_)                                                                        \
    {                                                                                                      \
        const int kb_ = (B_) - wbase(P);                   /* bit inside the register slot */              \
        const int s_ = LOGN - 1 - (B_);                    /* stage number of the transform */             \
        /* twiddle index = 2^s + (global index >> (b + 1)) */                                              \
        const uint32_t base_ = (1u << s_) + (blk << (LOGB - (B_) - 1)) + (hi << (ELOG - kb_ - 1));         \
        _Pragma("unroll") for (int g_ = 0; g_ < (E >> (kb_ + 1)); ++g_)                                    \
        {                                                                                                  \
            if constexpr (uniform_tw<P>()) DST[(OFF_) + g_] = A::load_u(tw, base_ + g_);                   \
            else DST[(OFF_) + g_] = A::load_v(tw, base_ + g_);                                             \
        }                                                                                                  \
    }

    // The whole set of pass P (nothing unless ahead<P>(); FOLD: the stage that multiplies by N^-1
    // takes none).  DESC: in the order a forward pass uses them (highest stage bit first).
    template <int P, bool FOLD, bool DESC>
    D2_DEV static void load_tw(Twid (&w)[E], int tid, uint32_t blk, const Tw *tw)
    {
        if constexpr (ahead<P>()) {
            constexpr int wb = wbase(P), lo = sbit(P), r = stages(P);
            const uint32_t hi = tw_hi<P>(tid);
#pragma unroll
            for (int i = 0; i < r; ++i) {
                const int b = DESC ? lo + r - 1 - i : lo + i;
                if (FOLD && b == LOGN - 1) continue;
                D2_LOAD_STAGE(w, tw_slot(b - wb, 0), b)
            }
        }
    }

    // SKIP_FIRST: the first stage of the pass has been done already (see forward_chained_small)
    template <int P, bool SKIP_FIRST = false>
    D2_DEV static void fwd_pass(elem (&x)[E], const Twid (&w)[E], int tid, uint32_t blk, const Tw *tw, const Mod &md)
    {
        constexpr int wb = wbase(P), lo = sbit(P), r = stages(P);
        const uint32_t hi = tw_hi<P>(tid);
        // Twiddles that are not fetched as a set (see ahead) are requested one stage ahead: those of the
        // next stage go out before the butterflies of this one, into the other of two small buffers.
        constexpr int first = lo + r - 1 - (SKIP_FIRST ? 1 : 0);
        Twid ws[2][E / 2 > 0 ? E / 2 : 1];
        if constexpr (!ahead<P>()) D2_LOAD_STAGE(ws[first & 1], 0, first)
#pragma unroll
        for (int b = first; b >= lo; --b) {           // stage bit inside the block index
            const int kb = b - wb;
            if constexpr (!ahead<P>()) {
                if (b > lo) {
                    D2_LOAD_STAGE(ws[(b - 1) & 1], 0, b - 1)
                    sched_fence();      // or the compiler moves the requests down to their first use
                }
            }
#pragma unroll
            for (int g = 0; g < (E >> (kb + 1)); ++g) {    // distinct twiddles of this stage
#pragma unroll
                for (int j = 0; j < (1 << kb); ++j) {
                    const int k0 = (g << (kb + 1)) | j;
                    if constexpr (ahead<P>())
                        A::template ct<uniform_tw<P>()>(x[k0], x[k0 | (1 << kb)], w[tw_slot(kb, g)], md);
                    else
                        A::template ct<uniform_tw<P>()>(x[k0], x[k0 | (1 << kb)], ws[b & 1][g], md);
                }
            }
        }
    }

    // FOLD: this pass contains the last stage of the whole inverse transform (bit LOGN-1)
    // and multiplies by N^-1 there: ninv = N^-1, wn = (inverse twiddle 1) * N^-1, both uniform over
    // the workgroup (they come from scalar loads of the per-modulus table).
    template <int P, bool FOLD>
    D2_DEV static void inv_pass(elem (&x)[E], const Twid (&w)[E], int tid, uint32_t blk, const Tw *tw, const Mod &md,
                                const Twid &ninv, const Twid &wn)
    {
        constexpr int wb = wbase(P), lo = sbit(P), r = stages(P);
        const uint32_t hi = tw_hi<P>(tid);
        if (P != NPASS - 1) {
#pragma unroll
            for (int k = 0; k < E; ++k) A::inv_pass_begin(x[k], md);
        }
        // stage-by-stage twiddles: one stage ahead, as in fwd_pass (the first stage's are requested here)
        Twid ws[2][E / 2 > 0 ? E / 2 : 1];
        if constexpr (!ahead<P>()) {
            if (!(FOLD && lo == LOGN - 1)) D2_LOAD_STAGE(ws[lo & 1], 0, lo)
        }
#pragma unroll
        for (int b = lo; b < lo + r; ++b) {
            const int kb = b - wb;
            if constexpr (!ahead<P>()) {
                if (b + 1 < lo + r && !(FOLD && b + 1 == LOGN - 1)) {
                    D2_LOAD_STAGE(ws[(b + 1) & 1], 0, b + 1)
                    sched_fence();
                }
            }
            if (FOLD && b == LOGN - 1) {
#pragma unroll
                for (int j = 0; j < (1 << kb); ++j) A::template gs_last<true>(x[j], x[j | (1 << kb)], ninv, wn, md);
            } else {
#pragma unroll
                for (int g = 0; g < (E >> (kb + 1)); ++g) {
#pragma unroll
                    for (int j = 0; j < (1 << kb); ++j) {
                        const int k0 = (g << (kb + 1)) | j;
                        if constexpr (ahead<P>())
                            A::template gs<uniform_tw<P>()>(x[k0], x[k0 | (1 << kb)], w[tw_slot(kb, g)], md);
                        else
                            A::template gs<uniform_tw<P>()>(x[k0], x[k0 | (1 << kb)], ws[b & 1][g], md);
                    }
                }
            }
        }
    }

    // LDS layout of an exchange between passes P and P+1 (either direction): one run of 2^W pad
    // words after every 2^(W + ELOG) coefficients, W = window base of pass P+1.  The side with the
    // large window touches runs of >= 32 consecutive words, the side with the small window walks
    // with a stride that the padding turns into 2^W (mod 32 words): both are conflict-free for
    // 8-byte accesses on 64 four-byte banks, 32 lanes per cycle pair.
    template <int X>   // X = the later pass of the pair
    D2_DEV static constexpr int phys_x(int idx)
    {
        constexpr int W = wbase(X);
        return idx + ((idx >> (W + ELOG)) << W);
    }
    // word of register slot k of thread tid in pass P = per-thread base + compile-time offset
    // (thread bits and slot bits of an index are disjoint, so the padded address splits).
    template <int P, int X>
    D2_DEV static int slot_base(int tid) { return phys_x<X>(index_of<P>(0, tid)); }
    template <int P, int X>
    static constexpr int slot_off(int k) { return phys_x<X>(k << wbase(P)); }

    // An exchange between two passes whose window bases are both <= 6 never leaves a wavefront:
    // the wave of a coefficient is then index >> (ELOG + 6) on both sides, and because every
    // exchange pads by the same ratio the words of wave v are [v, v + 1) * 64 * (E + 1) in all of
    // them.  Such an exchange needs no workgroup barrier (LDS serves the instructions of one wave
    // in order), only a guarantee that the compiler keeps the order.
    template <int PF, int PT>
    static constexpr bool intra_wave() { return wbase(PF < PT ? PF : PT) <= 6; }

    // Hand the coefficients from the owners of pass PF to the owners of pass PT.
    // FRESH: no wave can still be reading this buffer (the first exchange of a chained transform, see PINGPONG).
    template <int PF, int PT, bool FRESH = false>
    D2_DEV static void exchange(elem (&x)[E], uint64_t *lds, int tid)
    {
        constexpr int X = PF > PT ? PF : PT;
        constexpr bool INTRA = intra_wave<PF, PT>();
        // the same word layout for 8-byte and 4-byte words (a policy with 4-byte words uses the first half
        // of the buffer; the padding is conflict-free for either width)
        typedef typename A::word word;
        word *wr = (word *)lds + slot_base<PF, X>(tid);
        const word *rd = (const word *)lds + slot_base<PT, X>(tid);
        if (INTRA) wave_sync(); else if (!FRESH) __syncthreads();      // earlier readers of these words are done
#pragma unroll
        for (int k = 0; k < E; ++k) wr[slot_off<PF, X>(k)] = to_word<A>(x[k]);
        if (INTRA) wave_sync(); else __syncthreads();
#pragma unroll
        for (int k = 0; k < E; ++k) x[k] = from_word<A>(rd[slot_off<PT, X>(k)]);
    }

    template <int P, bool FRESH = false, bool SKIP_FIRST = false>
    D2_DEV static void fwd_from(elem (&x)[E], const Twid (&w)[E], uint64_t *lds, int tid, uint32_t blk,
                                const Tw *tw, const Mod &md)
    {
        if constexpr (P + 1 < NPASS) {
            Twid wn[E];
            fwd_pass<P, SKIP_FIRST>(x, w, tid, blk, tw, md);
            load_tw<P + 1, false, true>(wn, tid, blk, tw);
            exchange<P, P + 1, FRESH && P == 0>(x, lds, tid);      // later exchanges meet this transform's own readers
            fwd_from<P + 1, FRESH>(x, wn, lds, tid, blk, tw, md);
        } else {
            fwd_pass<P, SKIP_FIRST>(x, w, tid, blk, tw, md);
#pragma unroll
            for (int k = 0; k < E; ++k) A::fwd_end(x[k], md);
        }
    }

    template <int P, bool FOLD>
    D2_DEV static void inv_from(elem (&x)[E], const Twid (&w)[E], uint64_t *lds, int tid, uint32_t blk,
                                const Tw *tw, const Mod &md, const Twid &ninv, const Twid &wn)
    {
        if constexpr (P > 0) {
            Twid wnext[E];
            inv_pass<P, FOLD>(x, w, tid, blk, tw, md, ninv, wn);
            load_tw<P - 1, FOLD, false>(wnext, tid, blk, tw);
            exchange<P, P - 1>(x, lds, tid);
            inv_from<P - 1, FOLD>(x, wnext, lds, tid, blk, tw, md, ninv, wn);
        } else {
            inv_pass<P, FOLD>(x, w, tid, blk, tw, md, ninv, wn);
        }
    }

    // x: pass-0 ownership (policy's forward input range) -> last-pass ownership, lazy.
    // LDS protocol of a workgroup: whoever writes words that other waves may still be reading
    // puts a workgroup barrier in front of the write.  The first exchange of a forward transform
    // is of that kind and has its barrier; later ones stay inside the wave.
    D2_DEV static void forward(elem (&x)[E], uint64_t *lds, int tid, uint32_t blk, const Tw *tw, const Mod &md)
    {
        Twid w[E];
        load_tw<0, false, true>(w, tid, blk, tw);
        fwd_from<0>(x, w, lds, tid, blk, tw, md);
    }

    // The next forward transform of a chain (see PINGPONG); `lds` holds LDS_CHAIN_WORDS words.
    D2_DEV static void forward_chained(elem (&x)[E], uint64_t *lds, uint32_t &turn, int tid, uint32_t blk, const Tw *tw,
                                       const Mod &md)
    {
        Twid w[E];
        load_tw<0, false, true>(w, tid, blk, tw);
        fwd_from<0, PINGPONG>(x, w, next_buffer(lds, turn), tid, blk, tw, md);
    }

    // The next forward transform of a chain for a whole polynomial of small signed coefficients
    // (|v[k]| <= 32: ternary or centred-binomial samples), given as plain integers in pass-0 ownership.
    // Its first stage multiplies the twiddle by a small number: the policy does that without a modular
    // reduction and without first mapping the inputs into [0, q) (ct_small); the remaining stages are
    // the usual ones.  Needs at least two stages in the first pass and a whole-polynomial engine.
    D2_DEV static void forward_chained_small(const int32_t (&v)[E], elem (&x)[E], uint64_t *lds, uint32_t &turn, int tid,
                                             const Tw *tw, const Mod &md)
    {
        static_assert(LOGB == LOGN && stages(0) >= 2 && ahead<0>(), "shape without a separable first stage");
        Twid w[E];
        load_tw<0, false, true>(w, tid, 0, tw);
        constexpr int kb = ELOG - 1;                      // the first stage pairs slots k and k + E/2, one twiddle
#pragma unroll
        for (int j = 0; j < (1 << kb); ++j)
            A::template ct_small<uniform_tw<0>()>(v[j], v[j | (1 << kb)], x[j], x[j | (1 << kb)], w[tw_slot(kb, 0)], md);
        fwd_from<0, PINGPONG, true>(x, w, next_buffer(lds, turn), tid, 0, tw, md);
    }

    // All twiddles of one transform, for callers that run several transforms with the same table and
    // block id: fetched once, they stay in registers (scalar registers for the uniform passes).
    // Only for shapes whose passes all take their twiddles as a set.
    struct Twiddles {
        Twid w[NPASS][E];
    };
    template <int P = 0>
    static constexpr bool all_ahead() { return ahead<P>() && (P + 1 == NPASS || all_ahead<(P + 1 < NPASS ? P + 1 : P)>()); }

    template <bool INV, bool FOLD, int P = 0>
    D2_DEV static void load_all(Twiddles &t, int tid, uint32_t blk, const Tw *tw)
    {
        load_tw<P, FOLD, !INV>(t.w[P], tid, blk, tw);
        if constexpr (P + 1 < NPASS) load_all<INV, FOLD, P + 1>(t, tid, blk, tw);
    }

    template <int P = 0, bool FRESH = false>
    D2_DEV static void forward(elem (&x)[E], uint64_t *lds, int tid, const Twiddles &t, const Mod &md)
    {
        static_assert(ahead<P>(), "shape loads twiddles stage by stage");
        fwd_pass<P>(x, t.w[P], tid, 0, nullptr, md);
        if constexpr (P + 1 < NPASS) {
            exchange<P, P + 1, FRESH && P == 0>(x, lds, tid);
            forward<P + 1, FRESH>(x, lds, tid, t, md);
        } else {
#pragma unroll
            for (int k = 0; k < E; ++k) A::fwd_end(x[k], md);
        }
    }
    D2_DEV static void forward_chained(elem (&x)[E], uint64_t *lds, uint32_t &turn, int tid, const Twiddles &t,
                                       const Mod &md)
    {
        forward<0, PINGPONG>(x, next_buffer(lds, turn), tid, t, md);
    }

    template <bool FOLD, int P = NPASS - 1>
    D2_DEV static void inverse(elem (&x)[E], uint64_t *lds, int tid, const Twiddles &t, const Mod &md,
                               const Twid &ninv, const Twid &wn)
    {
        static_assert(ahead<P>(), "shape loads twiddles stage by stage");
        if constexpr (P == NPASS - 1 && NPASS > 1) {
            if (intra_wave<NPASS - 1, NPASS - 2>()) __syncthreads();
        }
        inv_pass<P, FOLD>(x, t.w[P], tid, 0, nullptr, md, ninv, wn);
        if constexpr (P > 0) {
            exchange<P, P - 1>(x, lds, tid);
            inverse<FOLD, P - 1>(x, lds, tid, t, md, ninv, wn);
        }
    }

    // x: last-pass ownership (canonical input) -> pass-0 ownership, lazy; scaled by N^-1 when FOLD.
    // The first exchange of an inverse transform stays inside the wave and therefore has no
    // barrier of its own: the one here covers readers in other waves (of staged inputs, or of the
    // last exchange of a preceding inverse transform).
    template <bool FOLD>
    D2_DEV static void inverse(elem (&x)[E], uint64_t *lds, int tid, uint32_t blk, const Tw *tw, const Mod &md,
                               const Twid &ninv, const Twid &wn)
    {
        Twid w[E];
        load_tw<NPASS - 1, FOLD, false>(w, tid, blk, tw);
        if constexpr (NPASS > 1) {
            if (intra_wave<NPASS - 1, NPASS - 2>()) __syncthreads();
        }
        inv_from<NPASS - 1, FOLD>(x, w, lds, tid, blk, tw, md, ninv, wn);
    }
};

}  // namespace d2
