"""CPU oracle of the lazy update (test infrastructure; see lpk_ref.c)."""
