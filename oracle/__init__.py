"""CPU oracle of the KVmix hot path. Test infrastructure only (see kvmix_ref.c)."""
