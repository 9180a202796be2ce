/*
 * prefix_cache.h: host-side prefix-cache bookkeeping for hybrid (attention + SSM)
 * models: a radix tree over token ids with judicious admission of SSM states
 * and FLOP-aware eviction (Sections 4.1 to 4.3, Eq. 1 and 2, Table 1).
 *
 * The library holds no model states.  It decides, for every request, from which
 * cached state the prefill can resume (hit_len, hit_handle: what ssm_prefill
 * takes as initial state), at which token position the prefill should checkpoint
 * a state (checkpoint_pos: what ssm_prefill takes as checkpoint position), and
 * which cached states must be released to stay within the capacity.  States are
 * named by caller-chosen non-negative 64-bit handles (for instance a slot index
 * in a device pool).  Everything here runs on the host; no GPU is involved.
 *
 * Not thread safe: calls on one cache must not overlap.  Errors are returned as
 * negative codes; pc_last_error() gives the thread's last message.
 */
#ifndef PREFIX_CACHE_H
#define PREFIX_CACHE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    PC_OK = 0,
    PC_ERR_INVALID_ARG = -1,   /* NULL pointer, negative size or handle                    */
    PC_ERR_BAD_REQUEST = -2,   /* pc_finish arguments do not match the tree or pc_begin    */
    PC_ERR_BUFFER_TOO_SMALL = -3
} pc_status_t;

/*
 * Model description for the FLOP efficiency of Eq. 1 (Table 1, FP16 states):
 * per layer and sequence length L, FLOPs of attention 8 L D^2 + 4 L^2 D, MLP
 * 16 L D^2, SSM 12 L D^2 + 16 L D N + 10 L; bytes of KVs 4 D per token and
 * attention layer, of an SSM state 2 D N (+ conv_state_bytes) per SSM layer.
 */
typedef struct {
    int32_t n_attn_layers;
    int32_t n_ssm_layers;
    int32_t n_mlp_layers;
    int32_t d_model;           /* D */
    int32_t d_state;           /* N */
    int64_t conv_state_bytes;  /* per SSM layer (Appendix A.1); 0 follows Table 1 */
    int64_t capacity_bytes;    /* cache budget for KVs and SSM states together */
    double alpha;              /* weight of FLOP efficiency in Eq. 2; 0 is LRU */
} pc_config_t;

typedef struct pc_cache pc_cache_t; /* opaque; owned by the library */

/* What a request may skip and what its prefill should checkpoint. */
typedef struct {
    int32_t hit_len;        /* leading input tokens that need no prefill; 0: none.  At most n - 1. */
    int32_t checkpoint_pos; /* prefix length (counted from the start of the sequence) whose state the
                               prefill should checkpoint, found by speculative insertion; 0: none */
    int64_t hit_handle;     /* handle of the state after hit_len tokens; -1 if hit_len is 0 */
} pc_lookup_t;

typedef struct {
    int64_t used_bytes;
    int64_t kv_tokens;  /* tokens whose KVs are cached */
    int64_t n_states;   /* cached SSM states */
    int64_t n_nodes;    /* radix-tree nodes without the root */
} pc_stats_t;

int pc_create(const pc_config_t *config, pc_cache_t **out);
void pc_destroy(pc_cache_t *cache);

/*
 * Before prefill (Section 4.1).  Finds the longest prefix of tokens[0..n) that
 * holds a cached state and is at most n - 1 long, refreshes that node's
 * timestamp (only that node's: Section 4.3) and pins it until pc_finish; then
 * inserts the input speculatively: if that would create a new intermediate node
 * (the input leaves the cached paths, or ends, in the middle of an edge) below
 * the hit, its depth is returned as checkpoint_pos.  The tree is not changed.
 * `now` is the caller's clock (any non-decreasing integer).
 */
int pc_begin(pc_cache_t *cache, const int32_t *tokens, int32_t n, int64_t now, pc_lookup_t *out);

/*
 * After the request has produced its last token.  tokens[0..m) is the whole
 * sequence, input and output; hit_len and checkpoint_pos are the values
 * pc_begin returned for it (the hit node is unpinned).  The sequence is
 * inserted, branch_handle (or -1) is attached as the state after
 * checkpoint_pos tokens and final_handle as the state after all m tokens (the
 * last decoded token is cached in any case).  Then nodes with at most one
 * child are evicted in the order of Eq. 2 until the cache fits its capacity;
 * the states of this request are exempt in this round.
 *
 * *n_evicted states were evicted and *n_rejected of the handles passed in were
 * not admitted because a state was already cached at that prefix; the caller
 * frees all of them and reads their handles with pc_released.
 */
int pc_finish(pc_cache_t *cache, const int32_t *tokens, int32_t m, int32_t hit_len, int32_t checkpoint_pos,
              int64_t branch_handle, int64_t final_handle, int64_t now, int32_t *n_evicted, int32_t *n_rejected);

/*
 * A request that pc_begin started and that will not reach pc_finish (it failed
 * or was cancelled) gives back the pin on its hit state here, so that the state
 * can be evicted again (Section 4.3: only states no request holds compete for
 * eviction).  tokens[0..hit_len) is the prefix pc_begin matched; hit_len 0 is
 * accepted and does nothing.  The tree and the timestamps are not changed.
 */
int pc_abort(pc_cache_t *cache, const int32_t *tokens, int32_t hit_len);

/*
 * Handles released by the last pc_finish: the evicted ones in eviction order,
 * then the rejected ones.  Copies them to out[0..) and returns their number,
 * or PC_ERR_BUFFER_TOO_SMALL (the list is kept) if cap is smaller.
 */
int pc_released(const pc_cache_t *cache, int64_t *out, int32_t cap);

int pc_stats(const pc_cache_t *cache, pc_stats_t *out);
int pc_set_alpha(pc_cache_t *cache, double alpha);
int pc_set_capacity(pc_cache_t *cache, int64_t capacity_bytes);

/* A deep copy (for replaying a window of requests under other settings: Section 4.2, "Managing the balance"). */
int pc_clone(const pc_cache_t *cache, pc_cache_t **out);

/* FLOPs of prefilling L tokens through all layers (Table 1), and the utility score S(n) of Eq. 2 of the node at
 * tokens[0..depth), for inspection and tests; PC_ERR_BAD_REQUEST if no state is cached there. */
double pc_prefill_flops(const pc_config_t *config, int64_t L);
int pc_node_score(const pc_cache_t *cache, const int32_t *tokens, int32_t depth, double *score);

const char *pc_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* PREFIX_CACHE_H */
