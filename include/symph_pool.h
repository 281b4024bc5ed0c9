/*
 * symph_pool.h - C ABI of the priority-ordered residency of K,V caches in HBM slots lent by the serving framework
 * (arxiv 2412.16434, Sec. 3.3: "priority-based K,V cache" and "cooperative memory management").  Host code only: no
 * call here touches a GPU; the transfers it decides on are carried out with the entry points of symph.h.
 *
 * What is modelled.  The cache memory is a pool of n_slots slots of one block (block_size tokens of one layer) each;
 * any slot can hold a block of any layer (address it through a symph_kv_cache view with n_layers = 1 and one block
 * table per session and layer).  A slot is free, owned by the framework, or lent to one layer of one announced
 * session ("unit": ceil(n_tokens / block_size) slots).  Symphony fills whatever the framework does not own, lower
 * layers first (the forward pass needs them first, the later ones arrive behind it), within a layer larger caches
 * first, then smaller session ids; units are held whole or not at all, one that does not fit is passed over.  When
 * the framework needs slots it first gets free ones and then overwrites lent units, later layers first, within a
 * layer the smallest cache first (the host copy stays valid, so giving a unit up moves no data).  With two announced
 * sessions and room for one, the lower layers of both are therefore held.
 *
 * Conventions: every pointer is a HOST pointer.  A pool is created by symph_pool_create, owned by the library until
 * symph_pool_destroy, and not thread-safe (serialise the calls on one pool).  Return values are symph_status codes
 * (symph.h); a call that fails changes nothing (SYMPH_ENOMEM aside: destroy the pool after it).  Slot numbers are
 * 0 .. n_slots-1; among free slots the lowest numbers are handed out first, so runs are reproducible.
 */
#ifndef SYMPH_POOL_H_
#define SYMPH_POOL_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct symph_pool symph_pool;

enum { SYMPH_POOL_EVICTED = 0, SYMPH_POOL_LOAD = 1 };

/* One entry of what symph_pool_settle reports. */
typedef struct {
  int64_t session;
  int32_t layer;
  int32_t kind;       /* SYMPH_POOL_EVICTED: the unit is no longer resident (its slots were freed or overwritten);
                         SYMPH_POOL_LOAD: the unit was given slots, unpack the layer into them */
  int32_t n_slots;    /* slots of the unit */
  int32_t slot_begin; /* LOAD: index of the unit's first slot in the slot array of the same call (block order:
                         token t goes to entry t / block_size); EVICTED: -1 */
} symph_pool_change;

/* n_layers, n_slots, block_size >= 1.  *out receives the pool. */
int32_t symph_pool_create(int32_t n_layers, int32_t n_slots, int32_t block_size, symph_pool** out);
void symph_pool_destroy(symph_pool* pool);

/* An advisory request (Sec. 3.1): session `session` with n_tokens >= 1 cached tokens is expected here.  Nothing moves
 * until symph_pool_settle.  Announcing a known session again with the same length is a no-op, with another length
 * SYMPH_EINVAL (drop it first). */
int32_t symph_pool_advise(symph_pool* pool, int64_t session, int32_t n_tokens);

/* The session will not be served here: its units are given up (reported by the next settle) and it is forgotten. */
int32_t symph_pool_drop(symph_pool* pool, int64_t session);

/* The session's request has arrived: its resident layers 0 .. r-1 pass to the framework as they are (no transfer) and
 * the session is forgotten.  h_slots receives r tables of ceil(n_tokens / block_size) slot numbers, layer after
 * layer; *n_resident_layers receives r.  SYMPH_EWORKSPACE if max_slots is too small (nothing changes; the need is
 * symph_pool_resident_layers * blocks). */
int32_t symph_pool_claim(symph_pool* pool, int64_t session, int32_t* h_slots, int32_t max_slots,
                         int32_t* n_resident_layers);

/* The framework takes n slots (memory pressure): free ones first, then lent units in the order stated above, whole
 * units at a time (what a unit leaves over becomes free).  h_slots [n] receives the slot numbers.  The evicted units
 * are reported by the next settle.  SYMPH_EWORKSPACE if fewer than n slots are not already the framework's. */
int32_t symph_pool_framework_take(symph_pool* pool, int32_t n, int32_t* h_slots);

/* The framework returns n slots it owns (SYMPH_EINVAL if one of them is not its own, or is listed twice). */
int32_t symph_pool_framework_give(symph_pool* pool, int32_t n, const int32_t* h_slots);

/* Bring the resident set to what the priorities say for the announced sessions and the slots the framework does not
 * own, and report every change since the last successful settle: first the units given up (by framework_take, drop
 * or this call), then the units to load, the most important first.  h_changes [max_changes], h_slots [max_slots].
 * *n_changes and *n_slots receive the counts written; if an array is too small they receive the counts needed,
 * nothing changes and the call returns SYMPH_EWORKSPACE. */
int32_t symph_pool_settle(symph_pool* pool, symph_pool_change* h_changes, int32_t max_changes, int32_t* h_slots,
                          int32_t max_slots, int32_t* n_changes, int32_t* n_slots);

/* Resident layers of an announced session (0 .. n_layers), or SYMPH_EINVAL if it is not known. */
int32_t symph_pool_resident_layers(const symph_pool* pool, int64_t session);

/* Slots per layer of an announced session, ceil(n_tokens / block_size), or SYMPH_EINVAL if it is not known. */
int32_t symph_pool_unit_slots(const symph_pool* pool, int64_t session);

/* The slots of one resident unit (its block table), h_slots [max_slots]; returns their number, SYMPH_EINVAL if the
 * unit is not resident, SYMPH_EWORKSPACE if max_slots is too small. */
int32_t symph_pool_table(const symph_pool* pool, int64_t session, int32_t layer, int32_t* h_slots, int32_t max_slots);

/* Slot counts by owner; any pointer may be null. */
int32_t symph_pool_counts(const symph_pool* pool, int32_t* n_free, int32_t* n_lent, int32_t* n_framework);

#ifdef __cplusplus
}
#endif
#endif /* SYMPH_POOL_H_ */
