"""Seeded synthetic inputs (token sequences -> keys -> sorted runs, trees, probe batches).

Input generation only: nothing here computes compaction, lookup or fence results.
"""
