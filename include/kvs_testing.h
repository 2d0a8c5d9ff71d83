/*
 * kvs_testing.h -- hooks of libkvs for its own tests and for tuning runs.  Not part of the
 * interface a serving stack builds on: nothing here is needed to use the library, and what is
 * here is process-wide state.
 */
#ifndef KVS_TESTING_H
#define KVS_TESTING_H

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Force the number of context tokens one workgroup of the split-context attention kernels
 * handles (a multiple of 64), so that small test cases run through many splits and their merge;
 * 0 restores the built-in choice, which sizes the splits to fill the GPU.  The setting is
 * process-wide and read by every later kvs_workspace_bytes() and attention call on every store
 * and thread: after changing it, query the workspace size again (a workspace sized under
 * another setting may be refused as too small; its contents stay valid, the counter region at
 * its start does not move).  Returns KVS_OK or KVS_ERR_INVALID_ARG.
 */
int kvs_testing_force_split_tokens(int tokens);

/*
 * Workgroups launched for a decode call that shares its pages out by tokens (0: the built-in
 * choice, one per compute unit; never fewer than the store has kv heads).  With a handful of
 * workgroups every share holds many sequences, and with thousands the shares are single octets,
 * which a test cannot arrange otherwise.  From 64 launched workgroups on, a launch over bf16 pages
 * of 128 channels with at least 24 octets per launched workgroup, whose shares are not whole
 * segments, lets only three quarters of them (a multiple of eight) take a share.  Process-wide;
 * query the workspace size again after changing it.
 */
int kvs_testing_set_decode_workgroups(int n);

/*
 * The integer plan by which a decode launch shares out its pages by tokens, as the kernel computes
 * it on the device, for a host-side check against brute force: a line of `total` octets (eight
 * pages each) is cut into n <= 65535 shares that differ by at most one octet, share i beginning at
 * octet floor(total * i / n) (a line shorter than n: one octet for each of the first workgroups).  kvs_testing_flat_share writes the share of workgroup i (first
 * octet, number of octets); kvs_testing_flat_owner returns the workgroup whose share holds octet
 * o, or -1 for arguments out of range.
 */
int kvs_testing_flat_share(int i, int n, int total, int* first, int* count);
int kvs_testing_flat_owner(int o, int n, int total);

#ifdef __cplusplus
}
#endif
#endif /* KVS_TESTING_H */
