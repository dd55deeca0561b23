// Floyd's subset algorithm with every slot resolved at once (one lane per slot).
//
// As written, slot j of a vertex with deg > F neighbors draws a candidate t_j in [0, deg-F+j] and takes it
// unless an earlier slot already holds that position, in which case it takes deg-F+j: the test is sequential
// over the slots.  Before slot i the chosen set is exactly {every earlier candidate} united with
// {deg-F+a for every earlier slot a that collided}, so slot i collides iff an earlier slot drew the same
// candidate, or its candidate equals deg-F+a for an earlier slot a that itself collided.  The second clause
// refers to a strictly earlier slot, so iterating it from "collides iff an earlier slot drew the same
// candidate" reaches its fixed point in at most F rounds.
//
// The rule is written against a small group interface so that the sampling kernel (lanes of a wavefront,
// shuffles) and a host-side lockstep harness (a CPU test that enumerates every candidate sequence) run the
// very same code:
//   candidate_of(j, mine)  the candidate of the group's slot j (every lane passes its own)
//   flag_of(j, mine)       the boolean `mine` of the group's slot j
//   any(b)                 true if b holds for any lane that takes part in the same exchange
#pragma once

#include <stdint.h>

#if defined(__HIPCC__)
#define ZG_FLOYD_FN __host__ __device__ __forceinline__
#else
#define ZG_FLOYD_FN inline
#endif

namespace zg {

// Position taken by slot `slot` of a vertex with `deg` neighbors and fanout F.  `active` lanes are slots of a
// vertex with deg > F (cand = their draw, in [0, deg-F+slot]); the other lanes of the group pass through with
// position = slot, and take part in the exchanges only as partners.
template <class Group>
ZG_FLOYD_FN uint32_t floyd_position(Group &grp, uint32_t slot, uint32_t F, uint32_t deg, bool active, uint32_t cand)
{
    const uint32_t tail0 = deg - F; // candidates >= tail0 coincide with the fallback position of slot cand - tail0
    bool dup = false;
    for (uint32_t j = 0; j + 1 < F; ++j) {
        const uint32_t cj = grp.candidate_of(j, cand);
        dup = dup || (j < slot && cj == cand);
    }
    dup = dup && active;
    const uint32_t a = cand - tail0; // meaningful only when cand >= tail0
    const bool chase = active && cand >= tail0 && a < slot;
    bool collide = dup;
    for (uint32_t it = 0; it < F; ++it) {
        const bool ca = grp.flag_of(chase ? a : 0u, collide);
        const bool nc = dup || (chase && ca);
        const bool changed = nc != collide;
        collide = nc;
        if (!grp.any(changed)) break;
    }
    return active ? (collide ? tail0 + slot : cand) : slot;
}

} // namespace zg
