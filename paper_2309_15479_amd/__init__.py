"""MI355X (gfx950) batched l2 LSH hash evaluation: FastLSH (sampled projection), dense
E2LSH on the matrix cores, sign hashes and compound-key packing, behind the C ABI of
``include/lsh.h``.  This package is only the Python binding (argument marshalling); all
hash arithmetic runs in the HIP kernels of ``liblsh.so`` (the collision-probability helpers
are host functions of the same library)."""
from .binding import (LshError, LshIndex, LshParams, candidate_offsets, e2lsh_collision_probability, equivalent_width,
                      fastlsh_collision_probability, fastlsh_moment_factors, hash_e2lsh, hash_fastlsh,
                      hash_fastlsh_keys, hash_fastlsh_ids_keys, hash_signs, library_path, load_library, pack_keys, pair_statistics,
                      project_e2lsh, project_fastlsh, time_launches, hash_mips_data, hash_mips_query,
                      mips_collision_probability, mips_kappa, project_mips_data, project_mips_query,
                      DENSE_AUTO, DENSE_FP32, DENSE_MATRIX)

__all__ = ["LshError", "LshIndex", "LshParams", "hash_e2lsh", "hash_fastlsh", "hash_fastlsh_keys", "hash_fastlsh_ids_keys", "hash_signs",
           "library_path", "load_library", "pack_keys", "project_e2lsh", "project_fastlsh",
           "time_launches", "e2lsh_collision_probability", "equivalent_width",
           "fastlsh_collision_probability", "fastlsh_moment_factors", "pair_statistics",
           "hash_mips_data", "hash_mips_query", "mips_collision_probability", "mips_kappa",
           "project_mips_data", "project_mips_query", "candidate_offsets", "DENSE_AUTO", "DENSE_FP32", "DENSE_MATRIX"]
