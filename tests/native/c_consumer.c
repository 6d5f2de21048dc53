/* A plain C99 consumer of the library's C ABI: includes the public header, starts a host-only
 * handle (no GPU), pushes a Write and the count Atomic that follows it through the ring exactly
 * as a kernel would, waits for the proxy, reads the statistics and the completion counter.
 * Built and run by tests/test_c_abi_from_c.py. */
#include <stdio.h>
#include <string.h>

#include "../../include/ep.h"

static uint32_t word0(uint32_t op, uint32_t src, uint32_t dst_rank, uint32_t local_expert) {
  return (op << 28) | (src << 20) | (dst_rank << 12) | local_expert;
}

int main(void) {
  ep_config c;
  ep_handle *h = NULL;
  ep_stats_t st;
  const int32_t *counts = NULL;
  uint64_t idx = 0;
  int rc;

  memset(&c, 0, sizeof c);
  c.num_ranks = 4;
  c.num_experts = 16;
  c.top_k = 2;
  c.hidden = 1024;
  c.max_tokens = 64;
  c.num_src = 1;
  c.num_channels = 2;
  c.ring_entries = 16;
  c.num_proxy_threads = 1;
  c.spin_timeout_ms = 5000;
  c.flags = EP_FLAG_HOST_ONLY;
  rc = ep_proxy_start(&c, &h);
  if (rc != EP_OK) {
    printf("start failed: %d (%s)\n", rc, ep_last_error());
    return 1;
  }
  /* compute calls refuse a handle without a GPU: there is no CPU fallback */
  if (ep_combine(h, NULL, NULL, NULL, 0, 0, NULL, NULL) != EP_ESTATE) return 2;
  if (ep_host_expect_atomics(h, 1) != EP_OK) return 3;
  /* one row of 2 KiB for expert 5 (rank 1, local expert 1), then its count */
  if (ep_host_push(h, 1, word0(EP_OP_WRITE, 0, 1, 1), 2048u >> 4, 0u, 0u, &idx) != EP_OK) return 4;
  if (ep_host_push(h, 1, word0(EP_OP_ATOMIC, 0, 1, 1), 1u, 0u, 0u * 4u + 1u, &idx) != EP_OK) return 5;
  rc = ep_wait(h);
  if (rc != EP_OK) {
    printf("wait failed: %d\n", rc);
    return 6;
  }
  if (ep_stats(h, &st) != EP_OK || ep_counters(h, &counts, NULL) != EP_OK) return 7;
  printf("cmds %lu writes %lu atomics_applied %lu rejected %lu count[5] %d\n", (unsigned long)st.cmds,
         (unsigned long)st.writes, (unsigned long)st.atomics_applied, (unsigned long)st.rejected, (int)counts[5]);
  if (st.cmds != 2 || st.writes != 1 || st.atomics_applied != 1 || st.rejected != 0 || counts[5] != 1) return 8;
  if (ep_proxy_stop(h) != EP_OK) return 9;
  return 0;
}
