/*
 * das_drafter.h -- host-side C ABI of the adaptive nonparametric drafter (Sec. 4.1.2 of the paper): a suffix-tree index
 * over a sliding window of recent rollouts, built online (Ukkonen's construction, linear time), queried for the longest match
 * between the end of the current context and the indexed rollouts, and read along the matched path for a chain draft.
 *
 * Plain host code: no device.  All pointers are host memory owned by the caller.  Tokens are int32 >= 0.
 * Every call returns DAS_DRAFTER_OK (0) or a negative code.  A das_drafter is not thread-safe.
 *
 * Window.  The index is a ring of at most `max_epochs` suffix trees, one per epoch (e.g. one RL iteration's rollouts of a
 * problem shard).  das_drafter_new_epoch opens a new tree and drops the oldest one when the ring is full: the drafter then
 * follows the policy as it drifts (Sec. 4.1.2).  Rollouts added with das_drafter_add go into the newest tree; a match never
 * spans two rollouts.
 *
 * Query.  For a context ctx[0..m), each tree gives the longest suffix of ctx (at most max_match tokens) that occurs in its
 * rollouts, in time linear in the tokens examined (suffix links, no restart per suffix).  The tree with the longest match
 * wins (ties: the newest).  The draft continues the match along the tree: inside an edge the next token is forced; at a
 * node the continuation that occurred most often is taken (ties: the smallest token), a rollout's end is never proposed.
 */
#ifndef DAS_DRAFTER_H
#define DAS_DRAFTER_H
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DAS_DRAFTER_OK            0
#define DAS_DRAFTER_ERR_INVALID  (-1)   /* null pointer, negative token or count, max_epochs < 1 */
#define DAS_DRAFTER_ERR_NOMEM    (-3)

typedef struct das_drafter das_drafter;

int das_drafter_create(int32_t max_epochs, das_drafter **out);
int das_drafter_free(das_drafter *d);
/* Open a new epoch (drops the oldest tree when max_epochs trees exist). */
int das_drafter_new_epoch(das_drafter *d);
/* Index one rollout (n >= 1 tokens) in the newest epoch.  Linear time overall. */
int das_drafter_add(das_drafter *d, const int32_t *tokens, int32_t n);
/* Longest match of the end of ctx[0..m) (looking at its last max_match tokens at most) and a chain draft of up to k tokens.
 * Writes the match length, the number of draft tokens (0 if the match is shorter than min_match) and the draft itself. */
int das_drafter_propose(das_drafter *d, const int32_t *ctx, int32_t m, int32_t max_match, int32_t min_match, int32_t k,
                        int32_t *match_len, int32_t *draft, int32_t *n_draft);
/* Indexed tokens and tree nodes over all live epochs. */
int das_drafter_size(das_drafter *d, int64_t *tokens, int64_t *nodes, int32_t *epochs);

#ifdef __cplusplus
}
#endif
#endif /* DAS_DRAFTER_H */
