"""CPU oracle for the segmented-gossip round: test infrastructure only.

Nothing in the product package may import this.  See combo_ref.cpp for what each
function follows in the paper.
"""
